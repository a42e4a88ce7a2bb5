// Software-pipelined sink+window attention kernel (same mathematics and cache layout as
// attn_kernel.hip; see there and kernels.h).
//
// A workgroup owns 256 queries of one head and streams the live kblocks of that head's
// K and V through an 8-stage LDS ring filled by direct-to-LDS loads.  Each wave owns
// QB blocks of 32 queries (QB = 1: 8 waves, two per SIMD; QB = 2: 4 waves, one per SIMD,
// every K/V fragment read from LDS feeds two MFMAs).
//
// Measured on gfx950: a 32x32x16 bf16 MFMA holds the matrix pipe for ~32 cycles; a lone
// wave issues a plain VALU instruction every ~5 cycles (two waves: one per ~2.5), exp2
// every ~9, packed bf16 convert / dot / max3 every ~4.5.  Both pipes stay busy only if
// every wave's own instruction stream mixes them finely, so a step (one kblock) is laid
// out as slots, each opened by one MFMA, with the vector work of the previous kblock in
// its shadow:
//     first  QB*KS   slots: S^T = K Q^T for kblock i+1
//     then   QB*2*DB slots: O^T += V^T P^T for kblock i
//     softmax numerators of kblock i as a skewed pipeline over the score pairs of a lane
//     (subtract reference | exp2 | pack to bf16 | add to row sum, one slot apart), the
//     running maximum of the new scores in the last slots, one LDS fragment read for
//     later use in every slot or every other slot.
// One workgroup barrier per step hands the ring stages over.
//
// VALU work is kept minimal: queries arrive pre-scaled by log2(e)/sqrt(D) (the append
// kernel folds that factor into the rotary epilogue) so p = exp2(s - m) with no
// multiply; row sums are taken over the bf16-rounded p (the values the second MFMA
// consumes) with the packed dot-product instruction.  The reference m moves only when
// a score exceeds it by more than RESCALE_SLACK (then O and the row sums are rescaled);
// the final division by the row sum makes the result independent of the reference.
#include "kernels.h"

namespace ll {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

constexpr float SP_RESCALE_SLACK = 6.0f;         // log2 units: p stays below 2^6 between rescales

__device__ __forceinline__ unsigned sp_pack_bf16(float a, float b) {
    f32x2 v = {a, b};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2));
}
// acc + lo + hi of a packed bf16 pair
__device__ __forceinline__ float sp_pair_sum(unsigned pair, float acc) {
    const bf16x2 one = {(__bf16)1.0f, (__bf16)1.0f};
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pair), one, acc, false);
}
// s_waitcnt that only waits for vector-memory loads: at most N outstanding.
template <int N>
__device__ __forceinline__ void sp_wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (0x7 << 4) | (0xF << 8));
}

// Up to three token-slot ranges are walked as one virtual list of kblocks: virtual index v lies
// in range 0 (v < n0), 1 (v < n01) or 2.  All arguments are plain scalars passed by value so
// that everything stays in scalar registers.
__device__ __forceinline__ int sp_pick(int v, int n0, int n01, int a0, int a1, int a2) {
    return v < n0 ? a0 : (v < n01 ? a1 : a2);
}
// Kblocks that may be cut by a range boundary are the first and last of each range; the one after v:
__device__ __forceinline__ int sp_next_edge(int v, int n0, int n01, int T) {
    const int cand[6] = {0, n0 - 1, n0, n01 - 1, n01, T - 1};
    int best = 0x7FFFFFFF;
#pragma unroll
    for (int c = 0; c < 6; ++c)
        if (cand[c] > v && cand[c] < best) best = cand[c];
    return best;
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

template <int D, int PF, int QB>
__device__ __forceinline__ void sp_attn_body(const AttnParams& p) {
    constexpr int KS = D / 16;                  // k-steps of S^T = K Q^T, also fragments per K kblock
    constexpr int DB = D / 32;                  // 32-row blocks of O^T
    constexpr int KB_BYTES = KBLOCK * D * 2;
    constexpr int STAGE_BYTES = 2 * KB_BYTES;   // [K kblock | V kblock]
    constexpr int NS = 8;                       // ring stages (a power of two: stage = kblock & 7)
    constexpr int NF = 2 * KS;                  // 1 KB fragments per stage
    constexpr int NW = 8 / QB;                  // waves per workgroup
    constexpr int LPW = NF / NW;                // loads per wave per kblock
    constexpr int QT = 256;
    static_assert(NF % NW == 0, "fragments must split over the waves");
    static_assert(PF >= 3, "kblock i + 2 must have landed when step i starts");
    static_assert(PF + 2 <= NS, "a stage is rewritten two barriers after its last read");

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
    const int q0 = ch.q_begin + (tile - ch.tile_begin) * QT + wave * (QB * 32);
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
    const int n0 = ke0 - kb0, n01 = n0 + (ke1 - kb1);                     // kblocks in range 0, in ranges 0 and 1
#define SP_PHYS_KB(v) ((v) + sp_pick((v), n0, n01, kb0, kb1 - n0, kb2 - n01))
#define SP_LIVE(v) sp_live_mask(SP_PHYS_KB(v) * KBLOCK, sp_pick((v), n0, n01, rs0, rs1, rs2), sp_pick((v), n0, n01, re0, re1, re2), half)

    // Q^T fragments (pre-scaled by log2(e)/sqrt(D)): fragment ks of block n holds features
    // 16*ks + 8*half + 0..7 of query q0 + 32n + col
    bf16x8 qf[QB][KS];
#pragma unroll
    for (int n = 0; n < QB; ++n) {
        const int row = min(q0 + n * 32 + col, q_end - 1);
        const uint16_t* src = p.q + (int64_t(row) * p.H + head) * D + half * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[n][ks] = *reinterpret_cast<const bf16x8*>(src + ks * 16);
    }

    const char* kbase = reinterpret_cast<const char*>(p.k_cache + head * p.head_stride);
    const char* vbase = reinterpret_cast<const char*>(p.v_cache + head * p.head_stride);

    // direct-to-LDS loads of physical kblock kb into a ring stage: one 1 KB fragment per instruction
    const unsigned lane_off = lane * 16;
    auto issue_loads = [&](int kb, int stage) {
        const int64_t kb_off = int64_t(kb) * KB_BYTES;
#pragma unroll
        for (int l = 0; l < LPW; ++l) {
            const int f = wave + NW * l;        // fragment of the stage this wave fetches
            const char* sbase = (f < KS ? kbase + f * 1024 : vbase + (f - KS) * 1024) + kb_off;   // wave-uniform
            const char* src = sbase + lane_off;
            char* dst = lds + stage * STAGE_BYTES + f * 1024;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src),
                                             (__attribute__((address_space(3))) void*)(dst), 16, 0, 0);
        }
    };

#pragma unroll
    for (int j = 0; j < PF; ++j) {
        const int v = min(j, T - 1);             // past the end the last kblock is fetched again, never used
        issue_loads(SP_PHYS_KB(v), j);
    }
    sp_wait_vmcnt<(PF - 3) * LPW>();            // this wave's loads of kblocks 0..2 have landed
    __builtin_amdgcn_s_barrier();

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
    auto mask_s = [&](f32x16& s, unsigned live) {
#pragma unroll
        for (int r = 0; r < 16; ++r)
            if (!((live >> r) & 1)) s[r] = -INFINITY;
    };
    auto max_s = [&](const f32x16& s) {
        float m = fmaxf(fmaxf(s[0], s[1]), s[2]);
#pragma unroll
        for (int r = 3; r < 15; r += 2) m = fmaxf(fmaxf(m, s[r]), s[r + 1]);
        return fmaxf(m, s[15]);
    };

    f32x16 o[QB][DB];
    float lsum[QB][2];                           // row sum of this lane's keys (two chains)
    float mref[QB];                              // reference maximum of this lane's query (log2 domain)
    f32x16 negm[QB];                             // every element = -mref: the score accumulators start from it
    float mx[QB];                                // largest score of kblock i among this lane's keys
    f32x16 sA[QB], sB[QB];                       // scores (log2 domain) of kblocks i and i + 1
    bf16x8 kfr[KS];                              // K fragments of kblock i + 1
    u32x4 vfr[2][DB];                            // V^T fragments of kblock i

    // ---- prologue: scores of kblock 0, the first reference, K fragments of kblock 1
    {
        const char* kt = lds + lane_off;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) kfr[ks] = *reinterpret_cast<const bf16x8*>(kt + ks * 1024);
    }
#pragma unroll
    for (int n = 0; n < QB; ++n) {
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[n][db][r] = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) sA[n][r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) sA[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr[ks], qf[n][ks], sA[n], 0, 0, 0);
        mask_s(sA[n], SP_LIVE(0));
        const float m = max_s(sA[n]);
        mref[n] = fmaxf(m, __shfl_xor(m, 32));  // a kblock of a range holds a live key: finite
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            negm[n][r] = -mref[n];
            sA[n][r] -= mref[n];
        }
        mx[n] = -INFINITY;
        lsum[n][0] = lsum[n][1] = 0.f;
    }
    {
        const char* kt = lds + (1 % NS) * STAGE_BYTES + lane_off;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) kfr[ks] = *reinterpret_cast<const bf16x8*>(kt + ks * 1024);
    }

    // ---- main loop, one kblock per step.  S_CUR holds the scores of kblock I on entry, S_NEXT those of
    // kblock I + 1 on exit; the loop alternates the two register sets so that no copy is needed.
    // Before the slots: the rare path (a score above the reference by more than the slack, or a kblock that
    // may be cut by a range boundary: mask, move the reference, rescale O and the sums).  A scheduling fence
    // after every slot keeps the compiler from regrouping the instructions and the empty asm statements pin
    // each stage's results inside its slot.  After the slots the wave waits for its own older loads and the
    // workgroup barrier hands the ring stages over.
    constexpr int QK_SLOTS = KS * QB, PV_SLOTS = 2 * DB * QB, NSLOT = QK_SLOTS + PV_SLOTS;
    constexpr int NPAIR = 8 * QB;                // score pairs per lane, in the order the second MFMA needs them
    constexpr int MAX_FIRST = NSLOT - 4 * QB;    // slots that take the maximum (the S^T chains have drained by then)
    // Pair j is word j % 4 of P^T fragment (query block (j / 4) % QB, key half j / (4 * QB)): the order in which
    // the second MFMA needs them.  The pairs are spread evenly over the slots before the last MFMA group that
    // needs them: pair j has its exp2 in slot j * SPAN / NPAIR, is packed one slot later and summed two slots
    // later, so every packed pair exists before the MFMA that consumes it.
    constexpr int SPAN = QK_SLOTS + DB * QB - 2;
    static_assert(((4 * QB - 1) * SPAN) / NPAIR + 1 <= QK_SLOTS - 1, "a packed pair would be late for its MFMA");
#define SP_PIN(x) asm volatile("" ::"v"(x))
#define SP_STEP(I, S_CUR, S_NEXT)                                                                                  \
    {                                                                                                               \
        const bool edge = (I) == next_edge;                                                                         \
        bool above = false;                                                                                         \
        _Pragma("unroll") for (int n = 0; n < QB; ++n) above = above || mx[n] > SP_RESCALE_SLACK;                   \
        if (edge || __any(above)) {                                                                                 \
            if (edge) next_edge = sp_next_edge((I), n0, n01, T);                                                    \
            _Pragma("unroll") for (int n = 0; n < QB; ++n) {                                                        \
                if (edge) {                                                                                         \
                    mask_s(S_CUR[n], SP_LIVE(I));                                                                   \
                    mx[n] = max_s(S_CUR[n]);                                                                        \
                }                                                                                                   \
                const float delta = fmaxf(fmaxf(mx[n], __shfl_xor(mx[n], 32)), 0.f);                                \
                const float alpha = __builtin_amdgcn_exp2f(-delta);                                                 \
                mref[n] += delta;                                                                                   \
                lsum[n][0] *= alpha;                                                                                \
                lsum[n][1] *= alpha;                                                                                \
                _Pragma("unroll") for (int db = 0; db < DB; ++db)                                                   \
                    _Pragma("unroll") for (int r = 0; r < 16; ++r) o[n][db][r] *= alpha;                            \
                _Pragma("unroll") for (int r = 0; r < 16; ++r) {                                                    \
                    negm[n][r] -= delta;                                                                            \
                    S_CUR[n][r] -= delta;                                                                           \
                }                                                                                                   \
            }                                                                                                       \
        }                                                                                                           \
        const char* vt = lds + (((I)) & (NS - 1)) * STAGE_BYTES + KB_BYTES + lane_off;                              \
        const char* kt = lds + (((I) + 2) & (NS - 1)) * STAGE_BYTES + lane_off;                                     \
        float d0[NPAIR], d1[NPAIR];                                                                                 \
        unsigned pb[QB][2][4];                                                                                      \
        float m_run[QB];                                                                                            \
        _Pragma("unroll") for (int n = 0; n < QB; ++n) m_run[n] = -INFINITY;                                        \
        _Pragma("unroll") for (int k = 0; k < NSLOT; ++k) {                                                         \
            if (k < QK_SLOTS) {                                                                                     \
                const int ks = k / QB, n = k % QB;                                                                  \
                S_NEXT[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr[ks], qf[n][ks], ks == 0 ? negm[n] : S_NEXT[n], 0, 0, 0); \
            } else {                                                                                                \
                const int g = (k - QK_SLOTS) / QB, n = (k - QK_SLOTS) % QB, t = g / DB, db = g % DB;                \
                const u32x4 bv = {pb[n][t][0], pb[n][t][1], pb[n][t][2], pb[n][t][3]};                              \
                o[n][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vfr[t][db]),          \
                                                                    __builtin_bit_cast(bf16x8, bv), o[n][db], 0, 0, 0); \
            }                                                                                                       \
            if (k == 0) {                                                                                           \
                const int v = min((I) + PF, T - 1);                                                                 \
                issue_loads(SP_PHYS_KB(v), ((I) + PF) & (NS - 1));                                                  \
            }                                                                                                       \
            _Pragma("unroll") for (int j = 0; j < NPAIR; ++j) {                                                     \
                const int n = (j / 4) % QB, t = j / (4 * QB), w = t * 4 + j % 4, e = (j * SPAN) / NPAIR;            \
                if (k == e) {                                                                                       \
                    d0[j] = __builtin_amdgcn_exp2f(S_CUR[n][2 * w]);                                                \
                    d1[j] = __builtin_amdgcn_exp2f(S_CUR[n][2 * w + 1]);                                            \
                    SP_PIN(d0[j]);                                                                                  \
                    SP_PIN(d1[j]);                                                                                  \
                }                                                                                                   \
                if (k == e + 1) {                                                                                   \
                    pb[n][t][j % 4] = sp_pack_bf16(d0[j], d1[j]);                                                   \
                    SP_PIN(pb[n][t][j % 4]);                                                                        \
                }                                                                                                   \
                if (k == e + 2) lsum[n][t] = sp_pair_sum(pb[n][t][j % 4], lsum[n][t]);                              \
            }                                                                                                       \
            if (k >= MAX_FIRST) {                                                                                   \
                const int n = (k - MAX_FIRST) / 4, r = ((k - MAX_FIRST) % 4) * 4;                                   \
                m_run[n] = fmaxf(fmaxf(m_run[n], S_NEXT[n][r]), S_NEXT[n][r + 1]);                                  \
                m_run[n] = fmaxf(fmaxf(m_run[n], S_NEXT[n][r + 2]), S_NEXT[n][r + 3]);                              \
            }                                                                                                       \
            if (k < QK_SLOTS) {                                                                                     \
                _Pragma("unroll") for (int f = 2 * k; f < 2 * k + 2; ++f)                                           \
                    if (f < 2 * DB)                                                                                 \
                        vfr[f / DB][f % DB] = *reinterpret_cast<const u32x4*>(vt + ((f % DB) * 2 + f / DB) * 1024); \
            } else {                                                                                                \
                _Pragma("unroll") for (int f = 2 * (k - QK_SLOTS); f < 2 * (k - QK_SLOTS) + 2; ++f)                 \
                    if (f < KS) kfr[f] = *reinterpret_cast<const bf16x8*>(kt + f * 1024);                           \
            }                                                                                                       \
            __builtin_amdgcn_sched_barrier(0);                                                                      \
            if (k == QK_SLOTS - 1 && edge) mask_v(vfr, SP_LIVE(I));                                                 \
        }                                                                                                           \
        _Pragma("unroll") for (int n = 0; n < QB; ++n) mx[n] = m_run[n];                                            \
        sp_wait_vmcnt<(PF - 3) * LPW>();                                                                            \
        __builtin_amdgcn_s_barrier();                                                                               \
    }

    int next_edge = 0;                           // next kblock that may be cut by a range boundary
    for (int i = 0; i < T; i += 2) {
        SP_STEP(i, sA, sB)
        if (i + 1 >= T) break;
        SP_STEP(i + 1, sB, sA)
    }
#undef SP_STEP
#undef SP_PIN
    sp_wait_vmcnt<0>();                          // nothing may still be writing LDS when the wave ends

    // out[row][head][32*db + 8*g + 4*half + i] = O^T register 4*g + i, divided by the row sum
#pragma unroll
    for (int n = 0; n < QB; ++n) {
        const float ls = lsum[n][0] + lsum[n][1];
        const float l = ls + __shfl_xor(ls, 32);
        const float inv = 1.0f / l;
        const int row = q0 + n * 32 + col;
        if (row < q_end) {
            uint16_t* dst = p.out + (int64_t(row) * p.H + head) * D + half * 4;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    u32x2 w = {sp_pack_bf16(o[n][db][4 * g] * inv, o[n][db][4 * g + 1] * inv),
                               sp_pack_bf16(o[n][db][4 * g + 2] * inv, o[n][db][4 * g + 3] * inv)};
                    *reinterpret_cast<u32x2*>(dst + db * 32 + g * 8) = w;
                }
        }
    }
#undef SP_PHYS_KB
#undef SP_LIVE
}

// QB = 1: 8 waves, two per SIMD (at most 256 VGPRs each).  QB = 2: 4 waves, one per SIMD (512 VGPRs).
template <int D, int PF>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2))) void ll_attn_sp1_kernel(const AttnParams p) {
    sp_attn_body<D, PF, 1>(p);
}
template <int D, int PF>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void ll_attn_sp2_kernel(const AttnParams p) {
    sp_attn_body<D, PF, 2>(p);
}

const AttnVariant kStreamVariants[] = {
    {"d128_sp1_pf4", 128, 256, 8 * 2 * KBLOCK * 128 * 2, ll_attn_sp1_kernel<128, 4>, 512},
    {"d128_sp1_pf6", 128, 256, 8 * 2 * KBLOCK * 128 * 2, ll_attn_sp1_kernel<128, 6>, 512},
    {"d64_sp1_pf4", 64, 256, 8 * 2 * KBLOCK * 64 * 2, ll_attn_sp1_kernel<64, 4>, 512},
};
const int kNumStreamVariants = sizeof(kStreamVariants) / sizeof(kStreamVariants[0]);

}  // namespace ll

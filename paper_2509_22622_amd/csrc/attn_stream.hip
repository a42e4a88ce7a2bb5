// Software-pipelined sink+window attention kernel (same mathematics and cache layout as
// attn_kernel.hip; see there and kernels.h).
//
// A workgroup of 8 waves (two per SIMD) owns 256 queries of one head, 32 per wave, and
// streams the live kblocks of that head's K and V through an 8-stage LDS ring filled by
// direct-to-LDS loads.  The workgroups of a head start together and walk its K/V in
// phase, so one copy of the stream in the XCD's L2 serves all of them.  (Cutting the
// launch into equal spans of kblocks per compute unit, to use the compute units that a
// tile count below their number leaves idle, was tried: workgroups at unrelated kblocks
// of a head each pull their own copy from HBM and the launch becomes bandwidth-bound;
// keeping the first kblocks of all tiles in phase and handing only the tails to the idle
// compute units costs more in partial results and merges than it gains.)
//
// Measured on gfx950 (two waves per SIMD, each an in-order stream): a 32x32x16 bf16 MFMA
// holds the matrix pipe for ~32 cycles; plain vector instructions issued behind an MFMA
// are free up to about two per MFMA and cost ~1 cycle each of matrix time beyond that;
// exp2 costs ~1 cycle; the packed dot-product instructions run on the matrix pipe and
// cost ~10 cycles each, so they are not used.  A step (one kblock) is laid out as slots,
// each opened by one MFMA, with the vector work of the previous kblock behind them:
//     first  KS   slots: S^T = K Q^T for kblock i+1
//     then   2*DB slots: O^T += V^T P^T for kblock i
//     softmax numerators of kblock i as a skewed pipeline over the score pairs of a lane
//     (exp2 | pack to bf16 and add to the row sum, one slot apart), the running maximum
//     of the new scores in the last slots, LDS fragment reads for later slots, and the
//     direct-to-LDS loads of a kblock six steps ahead.
// One workgroup barrier per two steps hands the ring stages over (lds_plan.h holds both hand-made
// synchronisation plans; host tests replay them).
//
// Under this load the chip is power-limited (its clock settles near 1.9 GHz with random bf16 operands): what
// counts is not only the matrix pipe's duty cycle but the energy spent next to it, hence no MFMAs for rows that
// do not exist, and the diagnostic kernel in probe_kernels.hip to measure the ceiling.
//
// Vector work is kept minimal: queries arrive pre-scaled by log2(e)/sqrt(D) (the append
// kernel folds that factor into the rotary epilogue) and the score accumulator starts at
// minus the reference, so p = exp2(s) with no subtract or multiply; row sums add the fp32
// p.  The reference m moves only when a score exceeds it by more than RESCALE_SLACK (then
// O and the row sums are rescaled); the final division by the row sum makes the result
// independent of the reference.
#include "kernels.h"
#include "lds_plan.h"

namespace ll {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

constexpr float SP_RESCALE_SLACK = 6.0f;         // log2 units: p stays below 2^6 between rescales
constexpr int SP_THREADS = 512;

__device__ __forceinline__ unsigned sp_pack_bf16(float a, float b) {
    f32x2 v = {a, b};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2));
}
// s_waitcnt that only waits for vector-memory loads: at most N outstanding.
template <int N>
__device__ __forceinline__ void sp_wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (0x7 << 4) | (0xF << 8));
}

// LDS reads the compiler does not see (it would wait for every outstanding read before the first use of any
// of them).  The read leaves `dst` pending; sp_lds_wait<N>(dst) must run before dst is used, N = reads issued
// after it by then (the LDS returns data in order, so "at most N outstanding" means this one has arrived).
__device__ __forceinline__ void sp_lds_read(u32x4& dst, unsigned addr, int offset) {
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(offset));
}
template <int N>
__device__ __forceinline__ void sp_lds_wait(u32x4& x) {
    asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(x) : "n"(N));
}
// the same for a count that is a constant only after unrolling; counts above the counter's range wait for 15
__device__ __forceinline__ void sp_lds_wait_n(u32x4& x, int n) {
    switch (n < 15 ? n : 15) {
        case 0: sp_lds_wait<0>(x); break;
        case 1: sp_lds_wait<1>(x); break;
        case 2: sp_lds_wait<2>(x); break;
        case 3: sp_lds_wait<3>(x); break;
        case 4: sp_lds_wait<4>(x); break;
        case 5: sp_lds_wait<5>(x); break;
        case 6: sp_lds_wait<6>(x); break;
        case 7: sp_lds_wait<7>(x); break;
        case 8: sp_lds_wait<8>(x); break;
        case 9: sp_lds_wait<9>(x); break;
        case 10: sp_lds_wait<10>(x); break;
        case 11: sp_lds_wait<11>(x); break;
        case 12: sp_lds_wait<12>(x); break;
        case 13: sp_lds_wait<13>(x); break;
        case 14: sp_lds_wait<14>(x); break;
        default: sp_lds_wait<15>(x); break;
    }
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

// Softmax state of the 32 queries of a wave after some of their kblocks: lane (col, half) holds, for query
// col, O^T rows 32*db + 8*(r/4) + 4*half + r%4 (unnormalised), the row sum over the keys this lane saw (the
// two halves of a column add up to the query's sum) and the reference both halves share.
template <int D>
struct SpState {
    f32x16 o[D / 32];
    float l, m;
};

// Virtual kblocks [vb, ve) of chunk `ch` for the 32 queries starting at row q0 of head `head`.
template <int D, bool QSCALE = false>
__device__ __forceinline__ void sp_segment(const AttnParams& p, const AttnChunk& ch, int head, int q0, int vb, int ve,
                                           char* lds, SpState<D>& st, const float2* shift_cs) {
    constexpr int KS = D / 16;                  // k-steps of S^T = K Q^T, also fragments per K kblock
    constexpr int DB = D / 32;                  // 32-row blocks of O^T
    constexpr int NV = 2 * DB;                  // V^T fragments per kblock
    constexpr int KB_BYTES = KBLOCK * D * 2;
    constexpr int STAGE_BYTES = 2 * KB_BYTES;   // [K kblock | V kblock]
    constexpr int NS = RingPlan::STAGES;        // ring stages (a power of two: stage = kblock & 7)
    constexpr int NF = KS + NV;                 // 1 KB fragments per stage
    constexpr int NW = 8;                       // waves per workgroup
    constexpr int LPW = NF / NW;                // direct-to-LDS loads per wave per kblock
    constexpr int PF = RingPlan::AHEAD;         // kblocks the loads run ahead
    constexpr int LAND = RingPlan::LANDED;      // kblocks that have landed when a pair of steps starts
    static_assert(NF % NW == 0, "fragments must split over the waves");
    // A pair of steps (i, i+1) reads kblocks i .. i+3; the barrier before it is passed only after every wave
    // has waited for its own loads of those kblocks.  The load issued in step j overwrites the stage of
    // kblock j + PF - NS, last read in step j + PF - NS, which lies before the barrier that precedes step j's pair.
    static_assert(PF >= LAND && PF + 2 <= NS, "ring too short for the prefetch distance");

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, kept in a scalar register
    const int col = lane & 31, half = lane >> 5;

    // ranges in scalar registers (no kernel-argument loads inside the loop)
    const int n_ranges = ch.n_ranges;
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

    // Q^T fragments (pre-scaled by log2(e)/sqrt(D)): fragment ks holds features 16*ks + 8*half + 0..7 of query q0 + col
    bf16x8 qf[KS];
    const uint16_t* q_src = p.q + (int64_t(min(q0 + col, q_end - 1)) * p.H + head) * D + half * 8;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[ks] = *reinterpret_cast<const bf16x8*>(q_src + ks * 16);
    if constexpr (QSCALE) {                     // queries that come as the model made them: fold the factor in here,
        const float c = p.scale_log2e;          // one rounding of the scaled value, as the append kernel does
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int j = 0; j < 8; ++j) qf[ks][j] = __bf16(float(qf[ks][j]) * c);
    }
    // Sink at a fixed rotary distance: range 0 is the sink, and its scores are taken with the queries turned back
    // by sink_shift frames on the frame axis: pair i (features 2i, 2i+1) times exp(-i * shift * freq_i), from the
    // table the workgroup prepared.  The scores of kblock v are computed one step ahead, so the unturned queries
    // are loaded again at the start of step n0 - 1 (the last kblock of range 0, always taken by the general step).
    const int sink_shift = ch.sink_shift;
    if (sink_shift != 0) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int pi = 8 * ks + 4 * half + j;
                if (pi < p.n_t) {
                    const float2 cs = shift_cs[pi];
                    const float re = float(qf[ks][2 * j]), im = float(qf[ks][2 * j + 1]);
                    qf[ks][2 * j] = __bf16(re * cs.x + im * cs.y);
                    qf[ks][2 * j + 1] = __bf16(im * cs.x - re * cs.y);
                }
            }
    }

    const char* kbase = reinterpret_cast<const char*>(p.k_cache + head * p.head_stride);
    const char* vbase = reinterpret_cast<const char*>(p.v_cache + head * p.head_stride);

    // direct-to-LDS load l of this wave for physical kblock kb into a ring stage: one 1 KB fragment
    const unsigned lane_off = lane * 16;
    const unsigned lds_a = (unsigned)(size_t)(__attribute__((address_space(3))) char*)lds + lane_off;   // LDS byte address
    auto issue_load = [&](int kb, int stage, int l) {
        const int64_t kb_off = int64_t(kb) * KB_BYTES;
        const int f = wave + NW * l;            // fragment of the stage this wave fetches
        const char* sbase = (f < KS ? kbase + f * 1024 : vbase + (f - KS) * 1024) + kb_off;   // wave-uniform
        const char* src = sbase + lane_off;
        char* dst = lds + stage * STAGE_BYTES + f * 1024;
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src),
                                         (__attribute__((address_space(3))) void*)(dst), 16, 0, 0);
    };

#pragma unroll
    for (int j = 0; j < PF; ++j) {
        const int v = min(vb + j, ve - 1);       // past the end the last kblock is fetched again, never used
#pragma unroll
        for (int l = 0; l < LPW; ++l) issue_load(SP_PHYS_KB(v), (vb + j) & (NS - 1), l);
    }
    sp_wait_vmcnt<(PF - LAND) * LPW>();         // this wave's loads of the first LAND kblocks have landed
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

    float lsum0, lsum1;                          // row sum of this lane's keys (two chains)
    float mref;                                  // reference maximum of this lane's query (log2 domain)
    f32x16 negm;                                 // every element = -mref: the score accumulators start from it
    float mx;                                    // largest score of kblock i among this lane's keys
    f32x16 sA, sB;                               // scores (log2 domain) of kblocks i and i + 1
    u32x4 kfr[KS];                               // K fragments of kblock i + 1
    u32x4 vfr[2][DB];                            // V^T fragments of kblock i

    // ---- prologue: scores of kblock vb, the first reference, K fragments of kblock vb + 1
    {
        const char* kt = lds + (vb & (NS - 1)) * STAGE_BYTES + lane_off;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) kfr[ks] = *reinterpret_cast<const u32x4*>(kt + ks * 1024);
    }
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) st.o[db][r] = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) sA[r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) sA = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kfr[ks]), qf[ks], sA, 0, 0, 0);
    mask_s(sA, SP_LIVE(vb));
    {
        const float m = max_s(sA);
        mref = fmaxf(m, __shfl_xor(m, 32));     // a kblock of a range holds a live key: finite
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        negm[r] = -mref;
        sA[r] -= mref;
    }
    mx = -INFINITY;
    lsum0 = lsum1 = 0.f;
    // the loop's first slots wait for these with the same counts as for the reads of a step before (reads the
    // compiler tracks would make it wait for everything at the loop head, in every iteration)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) sp_lds_read(kfr[ks], lds_a + ((vb + 1) & (NS - 1)) * STAGE_BYTES, ks * 1024);

    // ---- main loop, one kblock per step.  S_CUR holds the scores of kblock I on entry, S_NEXT those of
    // kblock I + 1 on exit; the loop alternates the two register sets so that no copy is needed.
    // Before the slots: the rare path (a score above the reference by more than the slack, or a kblock that
    // may be cut by a range boundary: mask, move the reference, rescale O and the sums).  A scheduling fence
    // after every slot keeps the compiler from regrouping the instructions and the empty asm statements pin
    // each stage's results inside its slot.  After every second step (odd index counted from vb) the wave waits
    // for its own older loads and the workgroup barrier hands the ring stages over.
    constexpr int NSLOT = KS + NV;
    constexpr int NPAIR = 8;                     // score pairs per lane, in the order the second MFMA needs them
    constexpr int MAX_FIRST = NSLOT - 4;         // slots that take the maximum (the S^T chain has drained by then)
    // Pair j is word j % 4 of the P^T fragment of key half j / 4.  The pairs are spread evenly over the slots
    // before the last MFMA group that needs them: pair j has its exp2 in slot j * SPAN / NPAIR and is packed and
    // summed one slot later, so every packed pair exists before the MFMA that consumes it.
    constexpr int SPAN = KS + DB - 2;
    static_assert((3 * SPAN) / NPAIR + 1 <= KS - 1, "a packed pair would be late for its MFMA");
    // The direct-to-LDS loads of a step are spread over its slots (back-to-back they stall the wave); the last
    // slot of each half measured best.
    constexpr int DMA_STEP = NSLOT / LPW, DMA_FIRST = DMA_STEP - 1;
    // Fragment reads and the waits before their use follow lds_plan.h.
    using Plan = LdsPlan<D>;
    static_assert(Plan::KS == KS && Plan::NV == NV, "plan and kernel disagree on the step's shape");
#define SP_PIN(x) asm volatile("" ::"v"(x))
#define SP_STEP(I, S_CUR, S_NEXT, EDGE, BAR)                                                                       \
    {                                                                                                               \
        const bool edge = EDGE && (I) == next_edge;                                                                 \
        if (__builtin_expect(edge || vote, 0)) {                                                                    \
            if (edge) {                                                                                             \
                next_edge = sp_next_edge((I), n0, n01, T);                                                          \
                mask_s(S_CUR, SP_LIVE(I));                                                                          \
                mx = max_s(S_CUR);                                                                                  \
                if (sink_shift != 0 && (I) == n0 - 1) {     /* the sink ends here: back to the unturned queries */  \
                    _Pragma("unroll") for (int ks = 0; ks < KS; ++ks)                                               \
                        qf[ks] = *reinterpret_cast<const bf16x8*>(q_src + ks * 16);                                 \
                }                                                                                                   \
            }                                                                                                       \
            const float delta = fmaxf(fmaxf(mx, __shfl_xor(mx, 32)), 0.f);                                          \
            const float alpha = __builtin_amdgcn_exp2f(-delta);                                                     \
            mref += delta;                                                                                          \
            lsum0 *= alpha;                                                                                         \
            lsum1 *= alpha;                                                                                         \
            _Pragma("unroll") for (int db = 0; db < DB; ++db)                                                       \
                _Pragma("unroll") for (int r = 0; r < 16; ++r) st.o[db][r] *= alpha;                                \
            _Pragma("unroll") for (int r = 0; r < 16; ++r) {                                                        \
                negm[r] -= delta;                                                                                   \
                S_CUR[r] -= delta;                                                                                  \
            }                                                                                                       \
        }                                                                                                           \
        const unsigned vt_a = lds_a + (((I)) & (NS - 1)) * STAGE_BYTES + KB_BYTES;                                  \
        const unsigned kt_a = lds_a + (((I) + 2) & (NS - 1)) * STAGE_BYTES;                                         \
        float d0[NPAIR], d1[NPAIR];                                                                                 \
        unsigned pb[2][4];                                                                                          \
        float m_run = -INFINITY;                                                                                    \
        _Pragma("unroll") for (int k = 0; k < NSLOT; ++k) {                                                         \
            /* the wave in its chain of dependent S^T MFMAs wins the issue arbitration against its SIMD partner */  \
            if (k == 0) __builtin_amdgcn_s_setprio(1);                                                              \
            if (k == KS) __builtin_amdgcn_s_setprio(0);                                                             \
            if (k < KS) {                                                                                           \
                sp_lds_wait_n(kfr[k], Plan::wait_k(k));                                                             \
                S_NEXT = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kfr[k]), qf[k],         \
                                                                  k == 0 ? negm : S_NEXT, 0, 0, 0);                 \
            } else {                                                                                                \
                const int g = k - KS, t = g / DB, db = g % DB;                                                      \
                const u32x4 bv = {pb[t][0], pb[t][1], pb[t][2], pb[t][3]};                                          \
                sp_lds_wait_n(vfr[t][db], Plan::wait_v(g));                                                         \
                st.o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vfr[t][db]),          \
                                                                    __builtin_bit_cast(bf16x8, bv), st.o[db], 0, 0, 0); \
            }                                                                                                       \
            if (k >= DMA_FIRST && (k - DMA_FIRST) % DMA_STEP == 0 && (k - DMA_FIRST) / DMA_STEP < LPW) {            \
                const int v = min((I) + PF, ve - 1);                                                                \
                issue_load(SP_PHYS_KB(v), ((I) + PF) & (NS - 1), (k - DMA_FIRST) / DMA_STEP);                       \
            }                                                                                                       \
            _Pragma("unroll") for (int j = 0; j < NPAIR; ++j) {                                                     \
                const int t = j / 4, e = (j * SPAN) / NPAIR;                                                        \
                if (k == e) {                                                                                       \
                    d0[j] = __builtin_amdgcn_exp2f(S_CUR[2 * j]);                                                   \
                    d1[j] = __builtin_amdgcn_exp2f(S_CUR[2 * j + 1]);                                               \
                    SP_PIN(d0[j]);                                                                                  \
                    SP_PIN(d1[j]);                                                                                  \
                }                                                                                                   \
                if (k == e + 1) {                                                                                   \
                    pb[t][j % 4] = sp_pack_bf16(d0[j], d1[j]);                                                      \
                    SP_PIN(pb[t][j % 4]);                                                                           \
                    lsum0 += d0[j];                                                                                 \
                    lsum1 += d1[j];                                                                                 \
                    SP_PIN(lsum0);                                                                                  \
                    SP_PIN(lsum1);                                                                                  \
                }                                                                                                   \
            }                                                                                                       \
            if (k >= MAX_FIRST) {                                                                                   \
                const int r = (k - MAX_FIRST) * 4;                                                                  \
                m_run = fmaxf(fmaxf(m_run, S_NEXT[r]), S_NEXT[r + 1]);                                              \
                m_run = fmaxf(fmaxf(m_run, S_NEXT[r + 2]), S_NEXT[r + 3]);                                          \
            }                                                                                                       \
            _Pragma("unroll") for (int f = 0; f < NV; ++f)                                                          \
                if (Plan::vslot(f) == k) sp_lds_read(vfr[f / DB][f % DB], vt_a, ((f % DB) * 2 + f / DB) * 1024);      \
            _Pragma("unroll") for (int f = 0; f < KS; ++f)                                                          \
                if (Plan::kslot(f) == k) sp_lds_read(kfr[f], kt_a, f * 1024);                                         \
            __builtin_amdgcn_sched_barrier(0);                                                                      \
            if (EDGE && k == KS - 1 && edge) {                                                                      \
                _Pragma("unroll") for (int f = 0; f < NV; ++f) sp_lds_wait<0>(vfr[f / DB][f % DB]);                 \
                mask_v(vfr, SP_LIVE(I));                                                                            \
            }                                                                                                       \
        }                                                                                                           \
        mx = m_run;                                                                                                 \
        vote = __any(mx > SP_RESCALE_SLACK);     /* decided here so that the next step opens with a scalar branch */ \
        if (BAR == 1 || (BAR == 2 && RingPlan::barrier_after((I) - vb))) {                                                           \
            sp_wait_vmcnt<(PF - LAND) * LPW>();                                                                     \
            __builtin_amdgcn_s_barrier();                                                                           \
        }                                                                                                           \
    }

    // Kblocks that a range boundary may cut (at most six per tile) take the general step, one at a time: it masks,
    // ends with the barrier when its index is odd, and hands the scores back in sA.  All others run in aligned
    // pairs through a step without any of that, so that the hot loop has one taken branch per two kblocks.
    int next_edge = sp_next_edge(vb - 1, n0, n01, T);   // next kblock that may be cut by a range boundary
    bool vote = false;                                   // some lane of the wave holds a score above the slack
    int i = vb;
    while (i < ve) {
        while (i < ve && (((i - vb) & 1) || i + 1 >= ve || i == next_edge || i + 1 == next_edge)) {
            SP_STEP(i, sA, sB, 1, 2)
            sA = sB;
            ++i;
        }
        for (int n = (min(ve, next_edge) - i) >> 1; n > 0; --n) {
            SP_STEP(i, sA, sB, 0, 0)
            SP_STEP(i + 1, sB, sA, 0, 1)
            i += 2;
        }
    }
#undef SP_STEP
#undef SP_PIN
#undef SP_PHYS_KB
#undef SP_LIVE
    __builtin_amdgcn_s_waitcnt(0);               // no load may still be writing LDS or registers past this point
    st.l = lsum0 + lsum1;
    st.m = mref;
}

// The part of sp_segment a wave without queries still owes its workgroup (the last tile of a chunk may have fewer
// than 256 rows): its share of the direct-to-LDS loads, with the same waits and the same number of barriers, and
// no arithmetic, which would only burn power on rows nobody reads.
template <int D>
__device__ __forceinline__ void sp_segment_loads_only(const AttnParams& p, const AttnChunk& ch, int head, int vb, int ve, char* lds) {
    constexpr int KS = D / 16, NV = D / 16;
    constexpr int KB_BYTES = KBLOCK * D * 2, STAGE_BYTES = 2 * KB_BYTES;
    constexpr int NS = RingPlan::STAGES, NW = 8, LPW = (KS + NV) / NW, PF = RingPlan::AHEAD, LAND = RingPlan::LANDED;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n_ranges = ch.n_ranges;
    const int rs0 = ch.rs[0], re0 = ch.re[0];
    int rs1 = ch.rs[1], re1 = ch.re[1], rs2 = ch.rs[2];
    if (n_ranges < 2) rs1 = re1 = 0;
    if (n_ranges < 3) rs2 = 0;
    const int kb0 = rs0 / KBLOCK, ke0 = (re0 + KBLOCK - 1) / KBLOCK;
    const int kb1 = rs1 / KBLOCK, ke1 = (re1 + KBLOCK - 1) / KBLOCK;
    const int kb2 = rs2 / KBLOCK;
    const int n0 = ke0 - kb0, n01 = n0 + (ke1 - kb1);
    const char* kbase = reinterpret_cast<const char*>(p.k_cache + head * p.head_stride);
    const char* vbase = reinterpret_cast<const char*>(p.v_cache + head * p.head_stride);
    const unsigned lane_off = lane * 16;
    auto issue_loads = [&](int v, int stage) {
        const int kb = v + sp_pick(v, n0, n01, kb0, kb1 - n0, kb2 - n01);
        const int64_t kb_off = int64_t(kb) * KB_BYTES;
#pragma unroll
        for (int l = 0; l < LPW; ++l) {
            const int f = wave + NW * l;
            const char* src = (f < KS ? kbase + f * 1024 : vbase + (f - KS) * 1024) + kb_off + lane_off;
            char* dst = lds + stage * STAGE_BYTES + f * 1024;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src),
                                             (__attribute__((address_space(3))) void*)(dst), 16, 0, 0);
        }
    };
#pragma unroll
    for (int j = 0; j < PF; ++j) issue_loads(min(vb + j, ve - 1), (vb + j) & (NS - 1));
    sp_wait_vmcnt<(PF - LAND) * LPW>();
    __builtin_amdgcn_s_barrier();
    for (int i = vb; i < ve; ++i) {
        issue_loads(min(i + PF, ve - 1), (i + PF) & (NS - 1));
        if (RingPlan::barrier_after(i - vb)) {   // the barrier that ends every second step of sp_segment
            sp_wait_vmcnt<(PF - LAND) * LPW>();
            __builtin_amdgcn_s_barrier();
        }
    }
    __builtin_amdgcn_s_waitcnt(0);
}

// out[row][head][32*db + 8*g + 4*half + i] = O^T register 4*g + i, divided by the row sum
template <int D>
__device__ __forceinline__ void sp_store_out(const AttnParams& p, int head, int q0, int q_end, const SpState<D>& st) {
    constexpr int DB = D / 32;
    const int lane = threadIdx.x & 63, col = lane & 31, half = lane >> 5;
    const float l = st.l + __shfl_xor(st.l, 32);
    const float inv = 1.0f / l;
    const int row = q0 + col;
    if (row < q_end) {
        uint16_t* dst = p.out + (int64_t(row) * p.H + head) * D + half * 4;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                u32x2 w = {sp_pack_bf16(st.o[db][4 * g] * inv, st.o[db][4 * g + 1] * inv),
                           sp_pack_bf16(st.o[db][4 * g + 2] * inv, st.o[db][4 * g + 3] * inv)};
                *reinterpret_cast<u32x2*>(dst + db * 32 + g * 8) = w;
            }
    }
}

// ---- one workgroup per (head, query tile)
template <int D, bool QSCALE, bool LSE = false>
__global__ __launch_bounds__(SP_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2))) void ll_attn_stream_kernel(const AttnParams p) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    __shared__ float2 shift_cs[64];              // (cos, sin) of sink_shift * frame-axis frequency, per rotary pair
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // Workgroups are dealt round-robin to the 8 XCDs, each with its own L2: the workgroups that stream the same
    // head's K/V should share one.
    const int xcd = blockIdx.x & 7;
    int idx = blockIdx.x >> 3, head = -1, tile = 0;
    if (p.n_groups == 0) {                       // one contiguous run of (head, tile) items per XCD
        // Runs of equal length (to within one item): XCD x takes items [ceil(x total / 8), ceil((x + 1) total / 8)).
        // With 12 heads of 19 tiles the cuts fall on a head boundary every second XCD, and the 12 heads make 16
        // (head, XCD) pairs, each streaming the head's K/V from memory once.
        const int total = p.n_tiles * p.H;
        const int item = ((xcd * total + 7) >> 3) + idx;
        if (item < (((xcd + 1) * total + 7) >> 3)) {
            head = item / p.n_tiles;
            tile = item % p.n_tiles;
        }
    } else {                                     // this XCD's list of (head, chunk) groups, longest tiles first
        for (int g = p.xcd_first[xcd]; g < p.xcd_first[xcd + 1]; ++g) {
            const int grp = p.xcd_group[g], c = grp % p.n_chunks;
            const int tiles = (c + 1 < p.n_chunks ? p.chunk[c + 1].tile_begin : p.n_tiles) - p.chunk[c].tile_begin;
            if (idx < tiles) {
                head = grp / p.n_chunks;
                tile = p.chunk[c].tile_begin + idx;
                break;
            }
            idx -= tiles;
        }
    }
    if (head < 0) return;                        // uniform over the workgroup
    int ci = 0;
    while (ci + 1 < p.n_chunks && tile >= p.chunk[ci + 1].tile_begin) ++ci;
    const AttnChunk& ch = p.chunk[ci];
    if (ch.sink_shift != 0) {                    // uniform over the workgroup
        if ((int)threadIdx.x < p.n_t) {
            double sn, cs;
            sincos(double(ch.sink_shift) * p.inv_freq_t[threadIdx.x], &sn, &cs);
            shift_cs[threadIdx.x] = make_float2(float(cs), float(sn));
        }
        __syncthreads();
    }
    // Waves w and w + 4 share a SIMD and take neighbouring 32-row blocks: in a chunk's short last tile the blocks
    // that do hold rows then pair up on SIMDs, and the workgroup advances at the pace of a full tile.  (One block
    // per SIMD would let it run some hundred kblocks ahead of the head's other workgroups, past what L2 keeps, and
    // the K/V it streamed would be fetched from memory a second time.)
    const int row_block = ((wave & 3) << 1) | (wave >> 2);
    const int q0 = ch.q_begin + (tile - ch.tile_begin) * 256 + row_block * 32;
    if (q0 >= ch.q_end) {                        // wave-uniform: this wave has no rows in the chunk's last tile
        sp_segment_loads_only<D>(p, ch, head, 0, ch.n_kblocks, lds);
        return;
    }
    SpState<D> st;
    sp_segment<D, QSCALE>(p, ch, head, q0, 0, ch.n_kblocks, lds, st, shift_cs);
    sp_store_out<D>(p, head, q0, ch.q_end, st);
    if constexpr (LSE) {                         // log2 of the row's sum of 2^score, for the backward pass
        const int lane = threadIdx.x & 63;
        const float l = st.l + __shfl_xor(st.l, 32);
        // v_log_f32 is the base-2 logarithm; callers that want no row sums leave the pointer null
        if (p.lse != nullptr && lane < 32 && q0 + lane < ch.q_end)
            p.lse[int64_t(head) * p.lse_stride + q0 + lane] = st.m + __builtin_amdgcn_logf(l);
        // and the output once more, not rounded to bf16: the backward pass takes delta = dO . O from it (with the
        // rounded output the error of delta, about 2^-9 |dO||O|, is what is left of dP - delta when one key holds
        // nearly all of a row's weight)
        if (p.out32 != nullptr && q0 + (lane & 31) < ch.q_end) {
            const float inv = 1.0f / l;
            float* dst = p.out32 + (int64_t(q0 + (lane & 31)) * p.H + head) * D + (lane >> 5) * 4;
#pragma unroll
            for (int db = 0; db < D / 32; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    typedef float f32x4 __attribute__((ext_vector_type(4)));
                    const f32x4 w = {st.o[db][4 * g] * inv, st.o[db][4 * g + 1] * inv, st.o[db][4 * g + 2] * inv, st.o[db][4 * g + 3] * inv};
                    *reinterpret_cast<f32x4*>(dst + db * 32 + g * 8) = w;
                }
        }
    }
}

const AttnVariant kStreamVariants[] = {
    {"d128_stream", 128, 256, 8 * 2 * KBLOCK * 128 * 2, ll_attn_stream_kernel<128, false>, SP_THREADS, KBLOCK},
    {"d64_stream", 64, 256, 8 * 2 * KBLOCK * 64 * 2, ll_attn_stream_kernel<64, false>, SP_THREADS, KBLOCK},
    // the same kernels for queries not yet multiplied by log2(e)/sqrt(D) (AttnParams::scale_log2e): cross-attention
    // over the prompt's keys, whose queries pass through no rotary step that could fold the factor in
    {"d128_stream_qscale", 128, 256, 8 * 2 * KBLOCK * 128 * 2, ll_attn_stream_kernel<128, true>, SP_THREADS, KBLOCK},
    {"d64_stream_qscale", 64, 256, 8 * 2 * KBLOCK * 64 * 2, ll_attn_stream_kernel<64, true>, SP_THREADS, KBLOCK},
    // the same kernels with one more output, the log2 of each row's sum of 2^score (AttnParams::lse): the forward of
    // the train-time rule, whose backward pass rebuilds the softmax weights from it
    {"d128_stream_lse", 128, 256, 8 * 2 * KBLOCK * 128 * 2, ll_attn_stream_kernel<128, false, true>, SP_THREADS, KBLOCK},
    {"d64_stream_lse", 64, 256, 8 * 2 * KBLOCK * 64 * 2, ll_attn_stream_kernel<64, false, true>, SP_THREADS, KBLOCK},
};
const int kNumStreamVariants = sizeof(kStreamVariants) / sizeof(kStreamVariants[0]);

}  // namespace ll

// The software-pipelined sink+window attention kernel of attn_stream.hip with both products on the 16x16x32 bf16
// MFMA instead of the 32x32x16 one (same mathematics, same cache layout in HBM, same LDS ring, same step plan).
//
// Why a second shape: under a full matrix load with real operand bits the chip is power-limited, and the 16x16x32
// instruction moves half as many accumulator bits per flop (a pure stream of them sustains about 13 % more than a
// stream of 32x32x16 MFMAs on the same chip).  A wave still owns 32 queries, now as two column blocks of 16, so every
// K or V^T fragment read from LDS feeds two MFMAs and the LDS traffic per flop is unchanged.
//
// Operand geometry (lane = 16 * g + n, g = 0..3, n = 0..15):
//   S^T block (m, qb) = K rows of key group m  x  queries 16 qb + n, contraction over 32 features per MFMA:
//       A: lane (g, n) holds A-row n, features 32 s + 8 g + 0..7;  B: query 16 qb + n, the same features;
//       C: lane (g, n) register j = A-row 4 g + j.
//     A-row r of key group m is taken from stored row (r & 7) + 8 m + 16 (r >> 3) of the K kblock (which holds key
//     swap23(row), see kernels.h), so that register j of lane (g, n) is key 8 g + 4 m + j: the eight scores a lane
//     holds for one query block are keys 8 g .. 8 g + 7 in the order (m, j).
//   O^T block (dq, qb) = V^T rows 16 dq + n  x  queries 16 qb + n, contraction over the kblock's 32 keys in ONE MFMA:
//       A: lane (g, n) holds feature 16 dq + n, keys 8 g + 0..7: one 16-byte piece of the V kblock as stored;
//       B: lane (g, n) holds keys 8 g + 0..7 of query 16 qb + n: exactly its own eight softmax weights.
//     So the weights never leave the lane here either.
// The K fragments are permuted on their way into LDS (direct-to-LDS loads take any 16 bytes of memory per lane but
// write lane l at offset 16 l): lane (c, m, r) of a load fetches stored row (r & 7) + 8 m + 16 (r >> 3) of 16-byte
// chunk c, which puts the 16 rows an MFMA's lane group reads side by side (no bank conflicts).
//
// A step (one kblock) keeps the 16 (D = 128) slots of attn_stream.hip, each now opened by the TWO MFMAs that share a
// fragment: K fragment k = (s = k / 2, m = k % 2) feeds S^T blocks (m, 0) and (m, 1); the O^T slots take the query
// block qb = 0 first (V^T fragments 2 j, 2 j + 1 in slot j), then qb = 1 with the same fragments again, so the
// weights of query block 0 are needed when the O^T slots begin and those of block 1 half way through them, as the
// two key halves were in the 32x32x16 form.  Exponentials, packing, row sums, the running maximum, fragment reads,
// direct-to-LDS loads, waits and barriers sit in the same slots (lds_plan.h: LdsPlan16, RingPlan).
#include "kernels.h"
#include "lds_plan.h"

namespace ll {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

constexpr float S16_RESCALE_SLACK = 6.0f;        // log2 units: p stays below 2^6 between rescales
constexpr int S16_THREADS = 512;
// Fixed-reference pass: a row sum above this (weights of 2^(score - reference), reference = largest score of the first
// kblock) sends the tile to the pass that follows the maximum.  Far below what fp32 sums and bf16 weights can hold.
constexpr float S16_FIXED_REF_LIMIT = 0x1p48f;

__device__ __forceinline__ unsigned s16_pack_bf16(float a, float b) {
    f32x2 v = {a, b};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2));
}
template <int N>
__device__ __forceinline__ void s16_wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (0x7 << 4) | (0xF << 8));
}
// LDS reads the compiler does not see; see attn_stream.hip.  The read leaves `dst` pending until s16_lds_wait<N>(dst)
// has run with N = reads issued after it by then.
__device__ __forceinline__ void s16_lds_read(u32x4& dst, unsigned addr, int offset) {
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(offset));
}
template <int N>
__device__ __forceinline__ void s16_lds_wait(u32x4& x) {
    asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(x) : "n"(N));
}
__device__ __forceinline__ void s16_lds_wait_n(u32x4& x, int n) {
    switch (n < 15 ? n : 15) {
        case 0: s16_lds_wait<0>(x); break;
        case 1: s16_lds_wait<1>(x); break;
        case 2: s16_lds_wait<2>(x); break;
        case 3: s16_lds_wait<3>(x); break;
        case 4: s16_lds_wait<4>(x); break;
        case 5: s16_lds_wait<5>(x); break;
        case 6: s16_lds_wait<6>(x); break;
        case 7: s16_lds_wait<7>(x); break;
        case 8: s16_lds_wait<8>(x); break;
        case 9: s16_lds_wait<9>(x); break;
        case 10: s16_lds_wait<10>(x); break;
        case 11: s16_lds_wait<11>(x); break;
        case 12: s16_lds_wait<12>(x); break;
        case 13: s16_lds_wait<13>(x); break;
        case 14: s16_lds_wait<14>(x); break;
        default: s16_lds_wait<15>(x); break;
    }
}
// a register that arrived together with (or before) one just waited for: only ties it to this point of the program
__device__ __forceinline__ void s16_lds_arrived(u32x4& x) { asm volatile("" : "+v"(x)); }

__device__ __forceinline__ int s16_pick(int v, int n0, int n01, int a0, int a1, int a2) {
    return v < n0 ? a0 : (v < n01 ? a1 : a2);
}
__device__ __forceinline__ int s16_next_edge(int v, int n0, int n01, int T) {
    const int cand[6] = {0, n0 - 1, n0, n01 - 1, n01, T - 1};
    int best = 0x7FFFFFFF;
#pragma unroll
    for (int c = 0; c < 6; ++c)
        if (cand[c] > v && cand[c] < best) best = cand[c];
    return best;
}
// bit e set: key key0 + 8 g + e (the e-th of the eight keys lane group g holds of a kblock) is inside [rs, re)
__device__ __forceinline__ unsigned s16_live_mask(int key0, int rs, int re, int g) {
    unsigned live = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int key = key0 + 8 * g + e;
        if (key >= rs && key < re) live |= 1u << e;
    }
    return live;
}

// Softmax state of the 32 queries of a wave: lane (g, n) holds, for query 16 qb + n, O^T rows 16 dq + 4 g + j
// (unnormalised), the row sum over the keys this lane saw (the four lane groups of a column add up to the query's
// sum) and the reference all four share.
template <int D>
struct S16State {
    f32x4 o[D / 16][2];
    float l[2], m[2];
};

// byte offset, inside a 1 KB K fragment as stored, of the 16 bytes that load lane `lane` fetches (see the file header)
__device__ __forceinline__ unsigned s16_k_load_offset(int lane) {
    const int c = lane >> 5, m = (lane >> 4) & 1, r = lane & 15;
    return unsigned(c * 32 + (r & 7) + 8 * m + 16 * (r >> 3)) * 16u;
}

// Virtual kblocks [vb, ve) of chunk `ch` for the 32 queries starting at row q0 of head `head`.
// SCHED selects where a step's vector and LDS work sits (bit 0: exponentials of the second query block moved behind
// the S^T slots; bit 1: one LDS fragment read per slot instead of two in half of the slots; bit 2: no issue priority)
// and, bit 3, whether the reference is fixed: the scores' running maximum is then not followed at all (no max3, no
// vote, no rescaling), the reference stays at the first kblock's maximum, and the caller must look at the row sums
// afterwards: a sum beyond S16_FIXED_REF_LIMIT (or not a number) means some score rose far above the reference, and
// the tile has to be computed again with the reference followed.
template <int D, bool QSCALE, int SCHED>
__device__ __forceinline__ void s16_segment(const AttnParams& p, const AttnChunk& ch, int head, int q0, int vb, int ve,
                                            char* lds, S16State<D>& st, const float2* shift_cs) {
    using Plan = LdsPlan16<D, (SCHED & 2) != 0>;
    constexpr bool TRACK = !(SCHED & 8);
    constexpr int KS = Plan::KS;                // K fragments per kblock = S^T slots (two MFMAs each)
    constexpr int NV = Plan::NV;                // V^T fragments per kblock = O^T slots (two MFMAs each)
    constexpr int NQ = D / 32;                  // contraction steps of S^T
    constexpr int HV = NV / 2;                  // O^T slots per query block
    constexpr int KB_BYTES = KBLOCK * D * 2;
    constexpr int STAGE_BYTES = 2 * KB_BYTES;   // [K kblock | V kblock]
    constexpr int NS = RingPlan::STAGES;
    constexpr int NF = KS + NV;                 // 1 KB fragments per stage
    constexpr int NW = 8;                       // waves per workgroup
    constexpr int LPW = NF / NW;                // direct-to-LDS loads per wave per kblock
    constexpr int PF = RingPlan::AHEAD;
    constexpr int LAND = RingPlan::LANDED;
    static_assert(NF % NW == 0, "fragments must split over the waves");
    static_assert(PF >= LAND && PF + 2 <= NS, "ring too short for the prefetch distance");

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, g = lane >> 4;

    const int n_ranges = ch.n_ranges;
    const int rs0 = ch.rs[0], re0 = ch.re[0];
    int rs1 = ch.rs[1], re1 = ch.re[1], rs2 = ch.rs[2], re2 = ch.re[2];
    if (n_ranges < 2) rs1 = re1 = 0;
    if (n_ranges < 3) rs2 = re2 = 0;
    const int kb0 = rs0 / KBLOCK, ke0 = (re0 + KBLOCK - 1) / KBLOCK;
    const int kb1 = rs1 / KBLOCK, ke1 = (re1 + KBLOCK - 1) / KBLOCK;
    const int kb2 = rs2 / KBLOCK, ke2 = (re2 + KBLOCK - 1) / KBLOCK;
    const int q_end = ch.q_end;
    const int T = (ke0 - kb0) + (ke1 - kb1) + (ke2 - kb2);
    const int n0 = ke0 - kb0, n01 = n0 + (ke1 - kb1);
#define S16_PHYS_KB(v) ((v) + s16_pick((v), n0, n01, kb0, kb1 - n0, kb2 - n01))
#define S16_LIVE(v) s16_live_mask(S16_PHYS_KB(v) * KBLOCK, s16_pick((v), n0, n01, rs0, rs1, rs2), s16_pick((v), n0, n01, re0, re1, re2), g)

    const char* kbase = reinterpret_cast<const char*>(p.k_cache + head * p.head_stride);
    const char* vbase = reinterpret_cast<const char*>(p.v_cache + head * p.head_stride);

    const unsigned lane_off = lane * 16;
    const unsigned k_load_off = s16_k_load_offset(lane);
    // LDS byte address of this lane's 16 bytes in fragment 0 of stage 0; fragment f of a kind adds s16_frag(f)
    const unsigned lds_a = (unsigned)(size_t)(__attribute__((address_space(3))) char*)lds + g * 512 + n * 16;
#define S16_FRAG(f) (((f) >> 1) * 2048 + ((f) & 1) * 256)
    auto issue_load = [&](int kb, int stage, int l) {
        const int64_t kb_off = int64_t(kb) * KB_BYTES;
        const int f = wave + NW * l;            // fragment of the stage this wave fetches (wave-uniform)
        const char* src = (f < KS ? kbase + f * 1024 + k_load_off : vbase + (f - KS) * 1024 + lane_off) + kb_off;
        char* dst = lds + stage * STAGE_BYTES + f * 1024;
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src),
                                         (__attribute__((address_space(3))) void*)(dst), 16, 0, 0);
    };

    // the ring's first loads go out before the queries are fetched: one memory latency for both
#pragma unroll
    for (int j = 0; j < PF; ++j) {
        const int v = min(vb + j, ve - 1);
#pragma unroll
        for (int l = 0; l < LPW; ++l) issue_load(S16_PHYS_KB(v), (vb + j) & (NS - 1), l);
    }

    // Q^T fragments (pre-scaled by log2(e)/sqrt(D)): fragment (qb, s) holds features 32 s + 8 g + 0..7 of query q0 + 16 qb + n
    bf16x8 qf[2][NQ];
    const uint16_t* q_src[2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        q_src[qb] = p.q + (int64_t(min(q0 + 16 * qb + n, q_end - 1)) * p.H + head) * D + g * 8;
#pragma unroll
        for (int s = 0; s < NQ; ++s) qf[qb][s] = *reinterpret_cast<const bf16x8*>(q_src[qb] + s * 32);
    }
    if constexpr ((SCHED & 16) != 0) {
        // the queries come as the model's projection made them: turn this lane's pairs (3D rotary embedding, the
        // frame axis from the table the cache write left, rows and columns from the cache's tables) and fold in the
        // softmax scale, with the arithmetic of the cache-write kernel (kernels.h: rope_turn_scaled)
        const int n_t = p.n_t, n_h = p.n_h;
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            const int rel = min(q0 + 16 * qb + n, q_end - 1) - ch.q_begin;
            const int fi = rel / p.P, tok = rel - fi * p.P;
            const int y = tok / p.grid_w, x = tok - y * p.grid_w;
            const float2* t_cs = p.t_table + (ch.t_row + fi) * MAX_T_PAIRS;
            const float2* r_cs = p.row_cs + y * n_h - n_t;
            const float2* c_cs = p.col_cs + x * p.n_w - n_t - n_h;
#pragma unroll
            for (int s = 0; s < NQ; ++s)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int pi = 16 * s + 4 * g + j;      // rotary pair of features 32 s + 8 g + 2 j, + 1
                    const float2 w = *(pi < n_t ? t_cs + pi : (pi < n_t + n_h ? r_cs + pi : c_cs + pi));
                    float re, im;
                    rope_turn_scaled(float(qf[qb][s][2 * j]), float(qf[qb][s][2 * j + 1]), w, p.q_scale, re, im);
                    qf[qb][s][2 * j] = __bf16(re);
                    qf[qb][s][2 * j + 1] = __bf16(im);
                }
        }
    }
    if constexpr (QSCALE) {
        const float c = p.scale_log2e;
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int s = 0; s < NQ; ++s)
#pragma unroll
                for (int j = 0; j < 8; ++j) qf[qb][s][j] = __bf16(float(qf[qb][s][j]) * c);
    }
    // Sink at a fixed rotary distance (see attn_stream.hip): range 0 is the sink, scored with the queries turned back
    // by sink_shift frames on the frame axis; the unturned queries are loaded again in step n0 - 1.
    const int sink_shift = ch.sink_shift;
    if (sink_shift != 0) {
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int s = 0; s < NQ; ++s)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int pi = 16 * s + 4 * g + j;      // rotary pair of features 32 s + 8 g + 2 j, + 1
                    if (pi < p.n_t) {
                        const float2 cs = shift_cs[pi];
                        const float re = float(qf[qb][s][2 * j]), im = float(qf[qb][s][2 * j + 1]);
                        qf[qb][s][2 * j] = __bf16(re * cs.x + im * cs.y);
                        qf[qb][s][2 * j + 1] = __bf16(im * cs.x - re * cs.y);
                    }
                }
    }

    s16_wait_vmcnt<(PF - LAND) * LPW>();
    __builtin_amdgcn_s_barrier();

    // dead slots may hold anything, even NaN: zero the V elements of keys outside the range
    auto mask_v = [&](u32x4 (&av)[NV], unsigned live) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const unsigned b0 = (live >> (2 * e)) & 1, b1 = (live >> (2 * e + 1)) & 1;
            const unsigned msk = (b0 ? 0x0000FFFFu : 0u) | (b1 ? 0xFFFF0000u : 0u);
#pragma unroll
            for (int f = 0; f < NV; ++f) av[f][e] &= msk;
        }
    };
    auto mask_s = [&](f32x4 (&s)[2][2], unsigned live) {
#pragma unroll
        for (int m = 0; m < 2; ++m)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (!((live >> (4 * m + j)) & 1)) {
                    s[m][0][j] = -INFINITY;
                    s[m][1][j] = -INFINITY;
                }
    };
    auto max_s = [&](const f32x4 (&s)[2][2], int qb) {
        float m = fmaxf(fmaxf(s[0][qb][0], s[0][qb][1]), s[0][qb][2]);
        m = fmaxf(fmaxf(m, s[0][qb][3]), s[1][qb][0]);
        m = fmaxf(fmaxf(m, s[1][qb][1]), s[1][qb][2]);
        return fmaxf(m, s[1][qb][3]);
    };
    // largest of the four lane groups that hold one query column
    auto col_max = [&](float x) {
        x = fmaxf(x, __shfl_xor(x, 16));
        return fmaxf(x, __shfl_xor(x, 32));
    };

    float lsum[2][2];                            // row sums of this lane's keys per query block (two chains each)
    float mref[2];                               // reference maximum per query block (log2 domain)
    f32x4 negm[2];                               // every element = -mref[qb]: the score accumulators start from it
    float mx[2];                                 // largest score of kblock i among this lane's keys, per query block
    f32x4 sA[2][2], sB[2][2];                    // scores [m][qb] (log2 domain) of kblocks i and i + 1
    u32x4 kfr[KS];                               // K fragments of kblock i + 1
    u32x4 vfr[NV];                               // V^T fragments of kblock i

    // ---- prologue: scores of kblock vb, the first reference, K fragments of kblock vb + 1
    {
        const char* kt = lds + (vb & (NS - 1)) * STAGE_BYTES + g * 512 + n * 16;
#pragma unroll
        for (int k = 0; k < KS; ++k) kfr[k] = *reinterpret_cast<const u32x4*>(kt + S16_FRAG(k));
    }
#pragma unroll
    for (int f = 0; f < NV; ++f)
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) st.o[f][qb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int m = 0; m < 2; ++m)
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) sA[m][qb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int k = 0; k < KS; ++k)
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
            sA[k & 1][qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kfr[k]), qf[qb][k >> 1], sA[k & 1][qb], 0, 0, 0);
    mask_s(sA, S16_LIVE(vb));
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        mref[qb] = col_max(max_s(sA, qb));       // a kblock of a range holds a live key: finite
        negm[qb] = f32x4{-mref[qb], -mref[qb], -mref[qb], -mref[qb]};
#pragma unroll
        for (int m = 0; m < 2; ++m) sA[m][qb] -= mref[qb];
        mx[qb] = -INFINITY;
        lsum[qb][0] = lsum[qb][1] = 0.f;
    }
#pragma unroll
    for (int k = 0; k < KS; ++k) s16_lds_read(kfr[k], lds_a + ((vb + 1) & (NS - 1)) * STAGE_BYTES, S16_FRAG(k));

    // ---- main loop: see attn_stream.hip for the plan; every slot here opens with two MFMAs
    constexpr int NSLOT = KS + NV;
    constexpr int NPAIR = 8;                     // score pairs per lane: pair j is word j % 4 of the P^T fragment of query block j / 4
    constexpr int MAX_FIRST = NSLOT - 4;
    constexpr int SPAN = KS + HV - 2;
    static_assert((3 * SPAN) / NPAIR + 1 <= KS - 1, "a packed pair would be late for its MFMA");
    static_assert(MAX_FIRST >= KS, "the running maximum would read scores still being accumulated");
    constexpr int DMA_STEP = NSLOT / LPW, DMA_FIRST = DMA_STEP - 1;
#define S16_PIN(x) asm volatile("" ::"v"(x))
#define S16_STEP(I, S_CUR, S_NEXT, EDGE, BAR)                                                                       \
    {                                                                                                               \
        const bool edge = EDGE && (I) == next_edge;                                                                 \
        if (__builtin_expect(edge || vote, 0)) {                                                                    \
            if (edge) {                                                                                             \
                next_edge = s16_next_edge((I), n0, n01, T);                                                         \
                mask_s(S_CUR, S16_LIVE(I));                                                                         \
                if (TRACK) {                                                                                        \
                    mx[0] = max_s(S_CUR, 0);                                                                        \
                    mx[1] = max_s(S_CUR, 1);                                                                        \
                }                                                                                                   \
                if (sink_shift != 0 && (I) == n0 - 1) {     /* the sink ends here: back to the unturned queries */  \
                    _Pragma("unroll") for (int qb = 0; qb < 2; ++qb)                                                \
                        _Pragma("unroll") for (int s = 0; s < NQ; ++s)                                              \
                            qf[qb][s] = *reinterpret_cast<const bf16x8*>(q_src[qb] + s * 32);                       \
                }                                                                                                   \
            }                                                                                                       \
            if (TRACK) _Pragma("unroll") for (int qb = 0; qb < 2; ++qb) {                                           \
                const float delta = fmaxf(col_max(mx[qb]), 0.f);                                                    \
                const float alpha = __builtin_amdgcn_exp2f(-delta);                                                 \
                mref[qb] += delta;                                                                                  \
                lsum[qb][0] *= alpha;                                                                               \
                lsum[qb][1] *= alpha;                                                                               \
                _Pragma("unroll") for (int f = 0; f < NV; ++f) st.o[f][qb] *= alpha;                                \
                negm[qb] -= delta;                                                                                  \
                S_CUR[0][qb] -= delta;                                                                              \
                S_CUR[1][qb] -= delta;                                                                              \
            }                                                                                                       \
        }                                                                                                           \
        const unsigned vt_a = lds_a + (((I)) & (NS - 1)) * STAGE_BYTES + KB_BYTES;                                  \
        const unsigned kt_a = lds_a + (((I) + 2) & (NS - 1)) * STAGE_BYTES;                                         \
        float d0[NPAIR], d1[NPAIR];                                                                                 \
        unsigned pb[2][4];                                                                                          \
        float m_run[2] = {-INFINITY, -INFINITY};                                                                    \
        _Pragma("unroll") for (int k = 0; k < NSLOT; ++k) {                                                         \
            if (k == 0 && !(SCHED & 4)) __builtin_amdgcn_s_setprio(1);                                              \
            if (k == KS && !(SCHED & 4)) __builtin_amdgcn_s_setprio(0);                                             \
            if (k < KS) {                                                                                           \
                const int m = k & 1, s = k >> 1;                                                                    \
                s16_lds_wait_n(kfr[k], Plan::wait_k(k));                                                            \
                S_NEXT[m][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kfr[k]), qf[0][s], \
                                                                        s == 0 ? negm[0] : S_NEXT[m][0], 0, 0, 0);  \
                S_NEXT[m][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kfr[k]), qf[1][s], \
                                                                        s == 0 ? negm[1] : S_NEXT[m][1], 0, 0, 0);  \
            } else {                                                                                                \
                const int qb = (k - KS) / HV, j = (k - KS) % HV;                                                    \
                const u32x4 bv = {pb[qb][0], pb[qb][1], pb[qb][2], pb[qb][3]};                                      \
                if (qb == 0) {                                                                                      \
                    s16_lds_wait_n(vfr[2 * j + 1], Plan::wait_v(j));                                                \
                    s16_lds_arrived(vfr[2 * j]);                                                                    \
                }                                                                                                   \
                st.o[2 * j][qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vfr[2 * j]),   \
                                      __builtin_bit_cast(bf16x8, bv), st.o[2 * j][qb], 0, 0, 0);                    \
                st.o[2 * j + 1][qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vfr[2 * j + 1]), \
                                          __builtin_bit_cast(bf16x8, bv), st.o[2 * j + 1][qb], 0, 0, 0);            \
            }                                                                                                       \
            if (k >= DMA_FIRST && (k - DMA_FIRST) % DMA_STEP == 0 && (k - DMA_FIRST) / DMA_STEP < LPW) {            \
                const int v = min((I) + PF, ve - 1);                                                                \
                issue_load(S16_PHYS_KB(v), ((I) + PF) & (NS - 1), (k - DMA_FIRST) / DMA_STEP);                      \
            }                                                                                                       \
            _Pragma("unroll") for (int j = 0; j < NPAIR; ++j) {                                                     \
                const int qb = j / 4, w = j % 4;                                                                    \
                const int e = !(SCHED & 1) ? (j * SPAN) / NPAIR                                                     \
                              : (qb == 0 ? (w * (KS - 1)) / 4 : KS - 1 + (w * (HV - 1)) / 3);                       \
                if (k == e) {                                                                                       \
                    d0[j] = __builtin_amdgcn_exp2f(S_CUR[w >> 1][qb][2 * (w & 1)]);                                 \
                    d1[j] = __builtin_amdgcn_exp2f(S_CUR[w >> 1][qb][2 * (w & 1) + 1]);                             \
                    S16_PIN(d0[j]);                                                                                 \
                    S16_PIN(d1[j]);                                                                                 \
                }                                                                                                   \
                if (k == e + 1) {                                                                                   \
                    pb[qb][w] = s16_pack_bf16(d0[j], d1[j]);                                                        \
                    S16_PIN(pb[qb][w]);                                                                             \
                    lsum[qb][0] += d0[j];                                                                           \
                    lsum[qb][1] += d1[j];                                                                           \
                    S16_PIN(lsum[qb][0]);                                                                           \
                    S16_PIN(lsum[qb][1]);                                                                           \
                }                                                                                                   \
            }                                                                                                       \
            if (TRACK && k >= MAX_FIRST) {                                                                          \
                const int qb = (k - MAX_FIRST) >> 1, m = (k - MAX_FIRST) & 1;                                       \
                m_run[qb] = fmaxf(fmaxf(m_run[qb], S_NEXT[m][qb][0]), S_NEXT[m][qb][1]);                            \
                m_run[qb] = fmaxf(fmaxf(m_run[qb], S_NEXT[m][qb][2]), S_NEXT[m][qb][3]);                            \
            }                                                                                                       \
            _Pragma("unroll") for (int f = 0; f < NV; ++f)                                                          \
                if (Plan::vslot(f) == k) s16_lds_read(vfr[f], vt_a, S16_FRAG(f));                                   \
            _Pragma("unroll") for (int f = 0; f < KS; ++f)                                                          \
                if (Plan::kslot(f) == k) s16_lds_read(kfr[f], kt_a, S16_FRAG(f));                                   \
            __builtin_amdgcn_sched_barrier(0);                                                                      \
            if (EDGE && k == KS - 1 && edge) {                                                                      \
                _Pragma("unroll") for (int f = 0; f < NV; ++f) s16_lds_wait<0>(vfr[f]);                             \
                mask_v(vfr, S16_LIVE(I));                                                                           \
            }                                                                                                       \
        }                                                                                                           \
        if (TRACK) {                                                                                                \
            mx[0] = m_run[0];                                                                                       \
            mx[1] = m_run[1];                                                                                       \
            vote = __any(fmaxf(mx[0], mx[1]) > S16_RESCALE_SLACK);                                                  \
        }                                                                                                           \
        if (BAR == 1 || (BAR == 2 && RingPlan::barrier_after((I) - vb))) {                                          \
            s16_wait_vmcnt<(PF - LAND) * LPW>();                                                                    \
            __builtin_amdgcn_s_barrier();                                                                           \
        }                                                                                                           \
    }

    int next_edge = s16_next_edge(vb - 1, n0, n01, T);
    bool vote = false;
    int i = vb;
    while (i < ve) {
        while (i < ve && (((i - vb) & 1) || i + 1 >= ve || i == next_edge || i + 1 == next_edge)) {
            S16_STEP(i, sA, sB, 1, 2)
#pragma unroll
            for (int m = 0; m < 2; ++m)
#pragma unroll
                for (int qb = 0; qb < 2; ++qb) sA[m][qb] = sB[m][qb];
            ++i;
        }
        for (int cnt = (min(ve, next_edge) - i) >> 1; cnt > 0; --cnt) {
            S16_STEP(i, sA, sB, 0, 0)
            S16_STEP(i + 1, sB, sA, 0, 1)
            i += 2;
        }
    }
#undef S16_STEP
#undef S16_PIN
#undef S16_PHYS_KB
#undef S16_LIVE
    __builtin_amdgcn_s_waitcnt(0);               // no load may still be writing LDS or registers past this point
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        st.l[qb] = lsum[qb][0] + lsum[qb][1];
        st.m[qb] = mref[qb];
    }
}

// A wave without queries (a chunk's short last tile) still owes its workgroup its share of the direct-to-LDS loads,
// with the same waits and the same number of barriers.
template <int D>
__device__ __forceinline__ void s16_segment_loads_only(const AttnParams& p, const AttnChunk& ch, int head, int vb, int ve, char* lds) {
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
    const unsigned lane_off = lane * 16, k_load_off = s16_k_load_offset(lane);
    auto issue_loads = [&](int v, int stage) {
        const int kb = v + s16_pick(v, n0, n01, kb0, kb1 - n0, kb2 - n01);
        const int64_t kb_off = int64_t(kb) * KB_BYTES;
#pragma unroll
        for (int l = 0; l < LPW; ++l) {
            const int f = wave + NW * l;
            const char* src = (f < KS ? kbase + f * 1024 + k_load_off : vbase + (f - KS) * 1024 + lane_off) + kb_off;
            char* dst = lds + stage * STAGE_BYTES + f * 1024;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src),
                                             (__attribute__((address_space(3))) void*)(dst), 16, 0, 0);
        }
    };
#pragma unroll
    for (int j = 0; j < PF; ++j) issue_loads(min(vb + j, ve - 1), (vb + j) & (NS - 1));
    s16_wait_vmcnt<(PF - LAND) * LPW>();
    __builtin_amdgcn_s_barrier();
    for (int i = vb; i < ve; ++i) {
        issue_loads(min(i + PF, ve - 1), (i + PF) & (NS - 1));
        if (RingPlan::barrier_after(i - vb)) {
            s16_wait_vmcnt<(PF - LAND) * LPW>();
            __builtin_amdgcn_s_barrier();
        }
    }
    __builtin_amdgcn_s_waitcnt(0);
}

// ---- one workgroup per (head, query tile): placement on the XCDs as in attn_stream.hip
template <int D, bool QSCALE, bool LSE, int SCHED = 0>
__global__ __launch_bounds__(S16_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2))) void ll_attn_stream16_kernel(const AttnParams p) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    __shared__ float2 shift_cs[64];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int xcd = blockIdx.x & 7;
    int idx = blockIdx.x >> 3, head = -1, tile = 0;
    if (p.n_groups == 0) {
        const int total = p.n_tiles * p.H;
        const int item = ((xcd * total + 7) >> 3) + idx;
        if (item < (((xcd + 1) * total + 7) >> 3)) {
            head = item / p.n_tiles;
            tile = item % p.n_tiles;
        }
    } else {
        for (int gi = p.xcd_first[xcd]; gi < p.xcd_first[xcd + 1]; ++gi) {
            const int grp = p.xcd_group[gi], c = grp % p.n_chunks;
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
    const int row_block = ((wave & 3) << 1) | (wave >> 2);      // waves w and w + 4 (one SIMD) take neighbouring blocks
    const int q0 = ch.q_begin + (tile - ch.tile_begin) * 256 + row_block * 32;
    // wave-uniform: a wave without rows in the chunk's last tile only takes its share of the loads and barriers
    const bool has_rows = q0 < ch.q_end;
    S16State<D> st;
    if (has_rows) s16_segment<D, QSCALE, SCHED>(p, ch, head, q0, 0, ch.n_kblocks, lds, st, shift_cs);
    else s16_segment_loads_only<D>(p, ch, head, 0, ch.n_kblocks, lds);
    if constexpr ((SCHED & 8) != 0) {
        // the pass above kept its first reference: fine unless some row's sum ran away (a score far above the first
        // kblock's maximum); then the whole workgroup (the waves share the ring and its barriers) takes the tile again
        // with the reference followed.  The barrier inside the vote also ends every wave's reads of the first pass.
        const bool ran_away = has_rows && !(st.l[0] < S16_FIXED_REF_LIMIT && st.l[1] < S16_FIXED_REF_LIMIT);
        if (__syncthreads_or(ran_away)) {
            if (has_rows) s16_segment<D, QSCALE, SCHED & ~8>(p, ch, head, q0, 0, ch.n_kblocks, lds, st, shift_cs);
            else s16_segment_loads_only<D>(p, ch, head, 0, ch.n_kblocks, lds);
        }
    }
    if (!has_rows) return;

    // out[row][head][16 dq + 4 g + j] = O^T block (dq, qb) register j, divided by the row sum
    const int lane = threadIdx.x & 63, n = lane & 15, g = lane >> 4;
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        float l = st.l[qb];
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        const float inv = 1.0f / l;
        const int row = q0 + 16 * qb + n;
        if (row < ch.q_end) {
            if (p.out_frag != nullptr) {         // uniform: the output projection's operand, 1 KB per store instruction
                const int n_ksteps = p.H * (D / 32);
#pragma unroll
                for (int t = 0; t < D / 32; ++t) {
                    const f32x4 a = st.o[2 * t][qb], b = st.o[2 * t + 1][qb];
                    const u32x4 w = {s16_pack_bf16(a[0] * inv, a[1] * inv), s16_pack_bf16(a[2] * inv, a[3] * inv),
                                     s16_pack_bf16(b[0] * inv, b[1] * inv), s16_pack_bf16(b[2] * inv, b[3] * inv)};
                    *reinterpret_cast<u32x4*>(p.out_frag + op_frag_offset(row, head * (D / 32) + t, g, n_ksteps)) = w;
                }
                continue;
            }
            uint16_t* dst = p.out + (int64_t(row) * p.H + head) * D + g * 4;
#pragma unroll
            for (int dq = 0; dq < D / 16; ++dq) {
                const f32x4 o = st.o[dq][qb];
                u32x2 w = {s16_pack_bf16(o[0] * inv, o[1] * inv), s16_pack_bf16(o[2] * inv, o[3] * inv)};
                *reinterpret_cast<u32x2*>(dst + dq * 16) = w;
            }
            if constexpr (LSE) {                 // for the backward pass of the train-time rule (see attn_stream.hip)
                if (p.lse != nullptr && g == 0)
                    p.lse[int64_t(head) * p.lse_stride + row] = st.m[qb] + __builtin_amdgcn_logf(l);
                if (p.out32 != nullptr) {
                    float* d32 = p.out32 + (int64_t(row) * p.H + head) * D + g * 4;
#pragma unroll
                    for (int dq = 0; dq < D / 16; ++dq) *reinterpret_cast<f32x4*>(d32 + dq * 16) = st.o[dq][qb] * inv;
                }
            }
        }
    }
}

// Default schedule: exponentials of the second query block behind the S^T slots, and the reference kept fixed with
// the second, maximum-following pass as the fallback (SCHED 9).  The *_tracked variants follow the maximum throughout;
// the *_qrope variants (SCHED bit 4) take unrotated queries and turn them on load.
constexpr int S16_DEFAULT = 9, S16_TRACKED = 1;
#define S16_ENTRY(name, D, QS, LSE, SCHED) \
    {name, D, 256, 8 * 2 * KBLOCK * D * 2, ll_attn_stream16_kernel<D, QS, LSE, SCHED>, S16_THREADS, KBLOCK}
const AttnVariant kStream16Variants[] = {
    S16_ENTRY("d128_stream16", 128, false, false, S16_DEFAULT),
    S16_ENTRY("d64_stream16", 64, false, false, S16_DEFAULT),
    S16_ENTRY("d128_stream16_qscale", 128, true, false, S16_DEFAULT),
    S16_ENTRY("d64_stream16_qscale", 64, true, false, S16_DEFAULT),
    S16_ENTRY("d128_stream16_lse", 128, false, true, S16_DEFAULT),
    S16_ENTRY("d64_stream16_lse", 64, false, true, S16_DEFAULT),
    S16_ENTRY("d128_stream16_tracked", 128, false, false, S16_TRACKED),
    S16_ENTRY("d64_stream16_tracked", 64, false, false, S16_TRACKED),
    S16_ENTRY("d128_stream16_qrope", 128, false, false, S16_DEFAULT | 16),
    S16_ENTRY("d64_stream16_qrope", 64, false, false, S16_DEFAULT | 16),
};
#undef S16_ENTRY
const int kNumStream16Variants = sizeof(kStream16Variants) / sizeof(kStream16Variants[0]);

}  // namespace ll

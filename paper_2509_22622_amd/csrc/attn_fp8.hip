// Sink+window attention over the 8-bit (E4M3) cache: the same key-set walk, LDS ring and workgroup shape as
// attn_stream.hip, with both products on the 32x32x64 fp8 MFMA.
//
// A workgroup of 8 waves owns 256 queries of one head, 32 per wave.  Per kblock of 64 keys a wave issues
//     2 * D/64 MFMAs   S^T = K8 Q8^T        (two 32-key row blocks, contraction over 64 features each)
//     D/32     MFMAs   O^T += V8^T P8^T     (contraction over the 64 keys)
// Every lane owns one query column: the 32 scores of a kblock that a lane holds in its two S^T accumulators are
// exactly the 32 contraction elements of its P8^T operand (the V8 image in the cache is permuted to that key
// order, kernels.h), so the softmax weights are converted to E4M3 in place with v_cvt_pk_fp8_f32 and never
// leave the lane.
//
// Numerics.  Queries arrive as E4M3 of q' * log2(e)/sqrt(D) * 2^k_exp and keys as E4M3 of K' * 2^-k_exp, so the
// accumulator holds the score in the log2 domain.  It starts at SHIFT - m (m = the lane's reference), and the
// weight is p = 2^(t - m + SHIFT): the reference maps to 2^SHIFT = 32 and, because the reference only moves
// when a score exceeds it by more than SLACK = 3, every weight stays below 2^8 = 256 < 448 (the largest E4M3
// value; the conversion does not saturate).  Weights 2^-6 .. 256 are normal E4M3 numbers: 14 binades below
// the largest score keep 3 mantissa bits, the 3 below those are subnormal, smaller ones round to zero.  Row
// sums add the fp32 weights before the conversion.  The final division by the row sum removes the reference
// and the shift; 2^v_exp is applied there.
//
// The scaled form of the MFMA is used with both scales 1 (E8M0 code 127).  The compiler may place its result on
// top of an operand that dies at the instruction, which this multi-pass instruction does not tolerate (wrong
// numbers, seen on the GPU): f8_mfma keeps both operands alive, together with the result, past the instruction, and
// tests/test_fp8_mfma_operands.py checks the generated code for such overlaps.  The same test checks that nothing
// is spilled: the hand-issued LDS reads below leave their destination registers pending, and a spill or copy of
// such a register before the counted wait would store stale data.
#include "kernels.h"
#include "lds_plan.h"

namespace ll {

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

constexpr float F8_SLACK = 3.0f;
constexpr float F8_SHIFT = 5.0f;
constexpr int F8_THREADS = 512;

__device__ __forceinline__ unsigned f8_pack_bf16(float a, float b) {
    f32x2 v = {a, b};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2));
}
template <int N>
__device__ __forceinline__ void f8_wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (0x7 << 4) | (0xF << 8));
}
__device__ __forceinline__ f32x16 f8_mfma(const i32x8& a, const i32x8& b, const f32x16& c) {
    f32x16 d = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 0, 0, 0, 0x7F7F7F7F, 0, 0x7F7F7F7F);
    // result and both operands are alive together here, after the instruction: the result cannot be placed on them
    asm volatile("" : "+v"(d) : "v"(a), "v"(b));
    return d;
}
__device__ __forceinline__ i32x8 f8_join(const u32x4& lo, const u32x4& hi) {
    i32x8 r = {int(lo[0]), int(lo[1]), int(lo[2]), int(lo[3]), int(hi[0]), int(hi[1]), int(hi[2]), int(hi[3])};
    return r;
}
__device__ __forceinline__ int f8_pick(int v, int n0, int n01, int a0, int a1, int a2) {
    return v < n0 ? a0 : (v < n01 ? a1 : a2);
}
__device__ __forceinline__ int f8_next_edge(int v, int n0, int n01, int T) {
    const int cand[6] = {0, n0 - 1, n0, n01 - 1, n01, T - 1};
    int best = 0x7FFFFFFF;
#pragma unroll
    for (int c = 0; c < 6; ++c)
        if (cand[c] > v && cand[c] < best) best = cand[c];
    return best;
}
// bit 16R + r set: the key of accumulator register r of row block R, for a lane in `half`, lies in [rs, re)
__device__ __forceinline__ unsigned f8_live_mask(int key0, int rs, int re, int half) {
    unsigned live = 0;
#pragma unroll
    for (int b = 0; b < 32; ++b) {
        const int key = key0 + 32 * (b >> 4) + 8 * ((b & 15) >> 2) + 4 * half + (b & 3);
        if (key >= rs && key < re) live |= 1u << b;
    }
    return live;
}

template <int D>
struct F8State {
    f32x16 o[D / 32];
    float l;
};

template <int D>
__device__ __forceinline__ void f8_segment(const AttnParams& p, const AttnChunk& ch, int head, int q0, char* lds, F8State<D>& st) {
    constexpr int DH = D / 64;                  // 64-feature halves: MFMAs per row block of S^T
    constexpr int DB = D / 32;                  // 32-row blocks of O^T
    constexpr int KB_BYTES = KBLOCK8 * D;       // one kblock of K (or of V)
    constexpr int STAGE_BYTES = 2 * KB_BYTES;   // [K kblock | V kblock]
    constexpr int NS = RingPlan::STAGES;
    constexpr int NF = STAGE_BYTES / 1024;      // 1 KB pieces per stage
    constexpr int NW = 8;
    constexpr int LPW = NF / NW;                // direct-to-LDS loads per wave per kblock
    constexpr int PF = RingPlan::AHEAD;
    constexpr int LAND = RingPlan::LANDED;
    static_assert(NF % NW == 0, "pieces must split over the waves");
    static_assert(PF >= LAND && PF + 2 <= NS, "ring too short for the prefetch distance");

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 31, half = lane >> 5;

    const int n_ranges = ch.n_ranges;
    const int rs0 = ch.rs[0], re0 = ch.re[0];
    int rs1 = ch.rs[1], re1 = ch.re[1], rs2 = ch.rs[2], re2 = ch.re[2];
    if (n_ranges < 2) rs1 = re1 = 0;
    if (n_ranges < 3) rs2 = re2 = 0;
    const int kb0 = rs0 / KBLOCK8, ke0 = (re0 + KBLOCK8 - 1) / KBLOCK8;
    const int kb1 = rs1 / KBLOCK8, ke1 = (re1 + KBLOCK8 - 1) / KBLOCK8;
    const int kb2 = rs2 / KBLOCK8, ke2 = (re2 + KBLOCK8 - 1) / KBLOCK8;
    const int q_end = ch.q_end;
    const int T = (ke0 - kb0) + (ke1 - kb1) + (ke2 - kb2);
    const int n0 = ke0 - kb0, n01 = n0 + (ke1 - kb1);
    const int vb = 0, ve = T;
#define F8_PHYS_KB(v) ((v) + f8_pick((v), n0, n01, kb0, kb1 - n0, kb2 - n01))
#define F8_LIVE(v) f8_live_mask(F8_PHYS_KB(v) * KBLOCK8, f8_pick((v), n0, n01, rs0, rs1, rs2), f8_pick((v), n0, n01, re0, re1, re2), half)

    // Q8^T operands: fragment dh holds features 64*dh + 32*half + 0..31 of query q0 + col
    i32x8 qf[DH];
    {
        const int row = min(q0 + col, q_end - 1);
        const uint8_t* src = p.q8 + (int64_t(row) * p.H + head) * D + half * 32;
#pragma unroll
        for (int dh = 0; dh < DH; ++dh)
            qf[dh] = f8_join(*reinterpret_cast<const u32x4*>(src + dh * 64), *reinterpret_cast<const u32x4*>(src + dh * 64 + 16));
    }

    const char* kbase = reinterpret_cast<const char*>(p.k8_cache + head * p.head_stride);
    const char* vbase = reinterpret_cast<const char*>(p.v8_cache + head * p.head_stride);
    const unsigned lane_off = lane * 16;
    auto issue_load = [&](int kb, int stage, int l) {
        const int64_t kb_off = int64_t(kb) * KB_BYTES;
        const int f = wave + NW * l;            // piece of the stage this wave fetches
        const char* sbase = (f < NF / 2 ? kbase + f * 1024 : vbase + (f - NF / 2) * 1024) + kb_off;   // wave-uniform
        const char* src = sbase + lane_off;
        char* dst = lds + stage * STAGE_BYTES + f * 1024;
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src),
                                         (__attribute__((address_space(3))) void*)(dst), 16, 0, 0);
    };

#pragma unroll
    for (int j = 0; j < PF; ++j) {
        const int v = min(vb + j, ve - 1);
#pragma unroll
        for (int l = 0; l < LPW; ++l) issue_load(F8_PHYS_KB(v), (vb + j) & (NS - 1), l);
    }
    f8_wait_vmcnt<(PF - LAND) * LPW>();
    __builtin_amdgcn_s_barrier();

    auto read_k = [&](int v, int R, int dh) {      // K8 operand (row block R, feature half dh) of virtual kblock v
        const char* kt = lds + (v & (NS - 1)) * STAGE_BYTES + ((R * DH + dh) * 2) * 1024 + lane_off;
        return f8_join(*reinterpret_cast<const u32x4*>(kt), *reinterpret_cast<const u32x4*>(kt + 1024));
    };
    auto read_v = [&](int v, int db) {             // V8^T operand (d-block db) of virtual kblock v
        const char* vt = lds + (v & (NS - 1)) * STAGE_BYTES + KB_BYTES + (db * 2) * 1024 + lane_off;
        return f8_join(*reinterpret_cast<const u32x4*>(vt), *reinterpret_cast<const u32x4*>(vt + 1024));
    };
    auto mask_s = [&](f32x16 (&s)[2], unsigned live) {
#pragma unroll
        for (int b = 0; b < 32; ++b)
            if (!((live >> b) & 1)) s[b >> 4][b & 15] = -INFINITY;
    };
    auto max_s = [&](const f32x16 (&s)[2]) {
        float m = fmaxf(s[0][0], s[1][0]);
#pragma unroll
        for (int r = 1; r < 16; ++r) m = fmaxf(fmaxf(m, s[0][r]), s[1][r]);
        return m;
    };

    float lsum0 = 0.f, lsum1 = 0.f;
    float mref;
    f32x16 negm;                                 // every element = SHIFT - mref
    float mx;                                    // largest accumulator value of kblock i among this lane's keys
    f32x16 sA[2], sB[2];

    // ---- prologue: scores of kblock vb and the first reference
    {
        float zero = 0.f;
        asm volatile("" : "+v"(zero));           // an accumulator input the compiler cannot fold into a constant
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) st.o[db][r] = 0.f;
#pragma unroll
        for (int R = 0; R < 2; ++R) {
#pragma unroll
            for (int r = 0; r < 16; ++r) sA[R][r] = zero;
#pragma unroll
            for (int dh = 0; dh < DH; ++dh) sA[R] = f8_mfma(read_k(vb, R, dh), qf[dh], sA[R]);
        }
        mask_s(sA, F8_LIVE(vb));
        const float m = max_s(sA);
        mref = fmaxf(m, __shfl_xor(m, 32));      // a kblock of a range holds a live key: finite
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            negm[r] = F8_SHIFT - mref;
            sA[0][r] += F8_SHIFT - mref;
            sA[1][r] += F8_SHIFT - mref;
        }
        mx = -INFINITY;
    }

    int next_edge = f8_next_edge(vb - 1, n0, n01, T);   // = vb: the first step masks kblock vb again (and its V operand)
    bool vote = false;

    // One step: scores of kblock I are in sC on entry, those of kblock I + 1 in sN on exit.
    auto step = [&](int I, f32x16 (&sC)[2], f32x16 (&sN)[2], bool barrier) {
        const bool v_edge = (I == next_edge);                        // kblock I may hold keys outside the range
        unsigned live = 0xFFFFFFFFu;
        if (__builtin_expect(v_edge || vote, 0)) {
            if (v_edge) {
                live = F8_LIVE(I);
                next_edge = f8_next_edge(I, n0, n01, T);
                mask_s(sC, live);
                mx = max_s(sC);
            }
            const float delta = fmaxf(fmaxf(mx, __shfl_xor(mx, 32)) - F8_SHIFT, 0.f);
            const float alpha = __builtin_amdgcn_exp2f(-delta);
            mref += delta;
            lsum0 *= alpha;
            lsum1 *= alpha;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) st.o[db][r] *= alpha;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                negm[r] -= delta;
                sC[0][r] -= delta;
                sC[1][r] -= delta;
            }
        }
        // direct-to-LDS loads of kblock I + PF
        {
            const int v = min(I + PF, ve - 1);
#pragma unroll
            for (int l = 0; l < LPW; ++l) issue_load(F8_PHYS_KB(v), (I + PF) & (NS - 1), l);
        }
        // S^T of kblock I + 1 (past the end: the ring holds the last kblock again, the result is never used)
#pragma unroll
        for (int R = 0; R < 2; ++R)
#pragma unroll
            for (int dh = 0; dh < DH; ++dh) sN[R] = f8_mfma(read_k(I + 1, R, dh), qf[dh], dh == 0 ? negm : sN[R]);
        // weights of kblock I
        i32x8 pb;
#pragma unroll
        for (int R = 0; R < 2; ++R)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const float e0 = __builtin_amdgcn_exp2f(sC[R][4 * g]), e1 = __builtin_amdgcn_exp2f(sC[R][4 * g + 1]);
                const float e2 = __builtin_amdgcn_exp2f(sC[R][4 * g + 2]), e3 = __builtin_amdgcn_exp2f(sC[R][4 * g + 3]);
                lsum0 += e0 + e2;
                lsum1 += e1 + e3;
                int w = __builtin_amdgcn_cvt_pk_fp8_f32(e0, e1, 0, false);
                w = __builtin_amdgcn_cvt_pk_fp8_f32(e2, e3, w, true);
                pb[R * 4 + g] = w;
            }
        // O^T += V8^T P8^T
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            i32x8 a = read_v(I, db);
            if (__builtin_expect(v_edge, 0)) {    // slots outside the range may hold anything, even NaN codes
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const unsigned b4 = (live >> (4 * j)) & 0xF;
                    const unsigned m = ((b4 & 1) ? 0xFFu : 0u) | ((b4 & 2) ? 0xFF00u : 0u) | ((b4 & 4) ? 0xFF0000u : 0u) | ((b4 & 8) ? 0xFF000000u : 0u);
                    a[j] &= int(m);
                }
            }
            st.o[db] = f8_mfma(a, pb, st.o[db]);
        }
        mx = max_s(sN);
        vote = __any(mx > F8_SHIFT + F8_SLACK);
        if (barrier) {
            f8_wait_vmcnt<(PF - LAND) * LPW>();
            __builtin_amdgcn_s_barrier();
        }
    };

    int i = vb;
    for (; i + 1 < ve; i += 2) {
        step(i, sA, sB, false);
        step(i + 1, sB, sA, true);
    }
    if (i < ve) step(i, sA, sB, false);
#undef F8_PHYS_KB
#undef F8_LIVE
    __builtin_amdgcn_s_waitcnt(0);
    st.l = lsum0 + lsum1;
}

// LDS reads the compiler does not see, with hand-counted waits (see f8_segment_sp).
__device__ __forceinline__ void f8_lds_read(u32x4& dst, unsigned addr, int offset) {
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(offset));
}
template <int N>
__device__ __forceinline__ void f8_lds_wait(u32x4& x, u32x4& y) {
    asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(x), "+v"(y) : "n"(N));
}

// The same computation as f8_segment as an explicit pipeline.  A step (one kblock of 64 keys) is NSLOT = D/16
// slots, each opened by one MFMA:
//     first  2*D/64 slots: S^T of kblock I + 1 (row block R, feature half dh), with the softmax weights of
//                          kblock I behind them (per slot: exp2 of 32/NK scores, their sum, their conversion
//                          to E4M3 into the P8^T operand);
//     then   D/32   slots: O^T += V8^T P8^T of kblock I, with the running maximum of the new scores behind them.
// Operand fragments (two 16-byte LDS reads each) are read two slots before their MFMA into four rotating
// register buffers (buffer = slot mod 4), so a read never lands in registers an MFMA issued less than two slots
// ago may still be reading.  The reads are inline asm; the LDS returns in order, and exactly one fragment (two
// reads) is issued between a fragment's own reads and its use, so every MFMA is preceded by s_waitcnt lgkmcnt(2).
// Ring, direct-to-LDS loads, waits and barriers are those of attn_stream.hip (lds_plan.h: a pair of steps reads
// kblocks i .. i+2 here, inside the i .. i+3 that plan covers).  Kblocks that a range boundary may cut run
// through the general form of the step one at a time, all others in aligned pairs through a form with no
// masking logic.
//
// LOGLIN = true is a cheaper way to the weights (the exponentials bound the exact form: 16 cycles each on the vector
// pipe).  An E4M3 code read as an integer is nearly linear in the logarithm of its value (8 codes per octave), so the
// code of 2^x is taken as round(8 x + 56) (56 = the code of 1.0) with one multiply-add and one v_cvt_pk_u8_f32 per
// score (which also clamps at 0 and inserts the byte into the operand word): the weight is 2^x times a factor between
// 0.96 and 1.02 (after the common factor has cancelled in the normalisation), on top of a rounding to an eighth of
// an octave.  The row sum is then taken from the same 8-bit weights by one more MFMA per kblock whose A operand is all
// ones, so numerator and denominator agree exactly and the output is a convex combination of the V8 rows; the
// accumulators hold the raw scores (started from zero), the reference enters through the multiply-add's constant.
template <int D, bool LOGLIN>
__device__ __forceinline__ void f8_segment_sp(const AttnParams& p, const AttnChunk& ch, int head, int q0, char* lds, F8State<D>& st) {
    constexpr int DH = D / 64;
    constexpr int DB = D / 32;
    constexpr int NK = 2 * DH;                  // S^T slots
    constexpr int NSLOT = NK + DB;
    constexpr int KB_BYTES = KBLOCK8 * D;
    constexpr int STAGE_BYTES = 2 * KB_BYTES;
    constexpr int NS = RingPlan::STAGES;
    constexpr int NF = STAGE_BYTES / 1024;
    constexpr int NW = 8;
    constexpr int LPW = NF / NW;
    constexpr int PF = RingPlan::AHEAD;
    constexpr int LAND = RingPlan::LANDED;
    constexpr int QPS = 8 / NK;                 // score quads converted per S^T slot
    constexpr int MPS = 32 / DB;                // scores entering the running maximum per O^T slot
    constexpr int DMA_STEP = NSLOT / LPW, DMA_FIRST = DMA_STEP - 1;
    using Plan = Fp8LdsPlan<D>;                 // which buffer a slot's fragment lives in, when it is read, the wait
    constexpr int AH = Plan::AHEAD_SLOTS;
    static_assert(Plan::NK == NK && Plan::NSLOT == NSLOT && Plan::BUFFERS == 4, "plan and kernel disagree on the step's shape");
    static_assert(NF % NW == 0 && 8 % NK == 0, "step shape");
    static_assert(PF >= LAND && PF + 2 <= NS, "ring too short for the prefetch distance");

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 31, half = lane >> 5;

    const int n_ranges = ch.n_ranges;
    const int rs0 = ch.rs[0], re0 = ch.re[0];
    int rs1 = ch.rs[1], re1 = ch.re[1], rs2 = ch.rs[2], re2 = ch.re[2];
    if (n_ranges < 2) rs1 = re1 = 0;
    if (n_ranges < 3) rs2 = re2 = 0;
    const int kb0 = rs0 / KBLOCK8, ke0 = (re0 + KBLOCK8 - 1) / KBLOCK8;
    const int kb1 = rs1 / KBLOCK8, ke1 = (re1 + KBLOCK8 - 1) / KBLOCK8;
    const int kb2 = rs2 / KBLOCK8, ke2 = (re2 + KBLOCK8 - 1) / KBLOCK8;
    const int q_end = ch.q_end;
    const int T = (ke0 - kb0) + (ke1 - kb1) + (ke2 - kb2);
    const int n0 = ke0 - kb0, n01 = n0 + (ke1 - kb1);
    const int vb = 0, ve = T;
#define F8_PHYS_KB(v) ((v) + f8_pick((v), n0, n01, kb0, kb1 - n0, kb2 - n01))
#define F8_LIVE(v) f8_live_mask(F8_PHYS_KB(v) * KBLOCK8, f8_pick((v), n0, n01, rs0, rs1, rs2), f8_pick((v), n0, n01, re0, re1, re2), half)

    i32x8 qf[DH];
    {
        const int row = min(q0 + col, q_end - 1);
        const uint8_t* src = p.q8 + (int64_t(row) * p.H + head) * D + half * 32;
#pragma unroll
        for (int dh = 0; dh < DH; ++dh)
            qf[dh] = f8_join(*reinterpret_cast<const u32x4*>(src + dh * 64), *reinterpret_cast<const u32x4*>(src + dh * 64 + 16));
    }

    const char* kbase = reinterpret_cast<const char*>(p.k8_cache + head * p.head_stride);
    const char* vbase = reinterpret_cast<const char*>(p.v8_cache + head * p.head_stride);
    const unsigned lane_off = lane * 16;
    const unsigned lds_a = (unsigned)(size_t)(__attribute__((address_space(3))) char*)lds + lane_off;
    auto issue_load = [&](int kb, int stage, int l) {
        const int64_t kb_off = int64_t(kb) * KB_BYTES;
        const int f = wave + NW * l;
        const char* sbase = (f < NF / 2 ? kbase + f * 1024 : vbase + (f - NF / 2) * 1024) + kb_off;
        const char* src = sbase + lane_off;
        char* dst = lds + stage * STAGE_BYTES + f * 1024;
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src),
                                         (__attribute__((address_space(3))) void*)(dst), 16, 0, 0);
    };

#pragma unroll
    for (int j = 0; j < PF; ++j) {
        const int v = min(vb + j, ve - 1);
#pragma unroll
        for (int l = 0; l < LPW; ++l) issue_load(F8_PHYS_KB(v), (vb + j) & (NS - 1), l);
    }
    f8_wait_vmcnt<(PF - LAND) * LPW>();
    __builtin_amdgcn_s_barrier();

    auto mask_s = [&](f32x16 (&s)[2], unsigned live) {
#pragma unroll
        for (int b = 0; b < 32; ++b)
            if (!((live >> b) & 1)) s[b >> 4][b & 15] = -INFINITY;
    };
    auto max_s = [&](const f32x16 (&s)[2]) {
        float m = fmaxf(s[0][0], s[1][0]);
#pragma unroll
        for (int r = 1; r < 16; ++r) m = fmaxf(fmaxf(m, s[0][r]), s[1][r]);
        return m;
    };

    float lsum0 = 0.f, lsum1 = 0.f;
    float mref;
    f32x16 negm;
    float mx;
    f32x16 sA[2], sB[2];
    f32x16 lacc;                                 // LOGLIN: row sums (every register of a lane holds its query's sum)
    i32x8 ones;                                  // LOGLIN: A operand of all 1.0
    float bias = 0.f;                            // LOGLIN: code of 2^(t - mref + SHIFT) = round(8 t + bias)
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    u32x4 fr[4][2];                              // rotating operand buffers: slot j uses fr[j % 4]
    unsigned vmask[8];                           // byte masks of the V8^T operand of a kblock cut by a range boundary

    // ---- prologue: scores of kblock vb and the first reference (plain reads: consumed here, nothing is pending
    // at the loop head), then the reads of the first two slots
    {
        float zero = 0.f;
        asm volatile("" : "+v"(zero));
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) st.o[db][r] = 0.f;
        const char* kt = lds + (vb & (NS - 1)) * STAGE_BYTES + lane_off;
#pragma unroll
        for (int R = 0; R < 2; ++R) {
#pragma unroll
            for (int r = 0; r < 16; ++r) sA[R][r] = zero;
#pragma unroll
            for (int dh = 0; dh < DH; ++dh) {
                const char* kp = kt + ((R * DH + dh) * 2) * 1024;
                sA[R] = f8_mfma(f8_join(*reinterpret_cast<const u32x4*>(kp), *reinterpret_cast<const u32x4*>(kp + 1024)), qf[dh], sA[R]);
            }
        }
        mask_s(sA, F8_LIVE(vb));
        const float m = max_s(sA);
        mref = fmaxf(m, __shfl_xor(m, 32));
        if (LOGLIN) {
            bias = 56.0f + 8.0f * (F8_SHIFT - mref);
#pragma unroll
            for (int r = 0; r < 16; ++r) lacc[r] = zero;
#pragma unroll
            for (int j = 0; j < 8; ++j) ones[j] = 0x38383838;
        } else {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                negm[r] = F8_SHIFT - mref;
                sA[0][r] += F8_SHIFT - mref;
                sA[1][r] += F8_SHIFT - mref;
            }
        }
        mx = -INFINITY;
#pragma unroll
        for (int j = 0; j < 8; ++j) vmask[j] = 0xFFFFFFFFu;
    }
    // fragment of slot j of the step whose S^T kblock is stage `ks` and whose O^T kblock is stage `vs`
#define F8_READ_FRAG(J, KT_A, VT_A)                                                                                 \
    {                                                                                                               \
        if ((J) < NK) {                                                                                             \
            f8_lds_read(fr[Plan::buffer(J)][0], (KT_A), ((J) * 2) * 1024);                                                  \
            f8_lds_read(fr[Plan::buffer(J)][1], (KT_A), ((J) * 2 + 1) * 1024);                                              \
        } else {                                                                                                    \
            f8_lds_read(fr[Plan::buffer(J)][0], (VT_A), (((J) - NK) * 2) * 1024);                                           \
            f8_lds_read(fr[Plan::buffer(J)][1], (VT_A), (((J) - NK) * 2 + 1) * 1024);                                       \
        }                                                                                                           \
    }
    {
        const unsigned kt_a = lds_a + ((vb + 1) & (NS - 1)) * STAGE_BYTES;
        const unsigned vt_a = lds_a + (vb & (NS - 1)) * STAGE_BYTES + KB_BYTES;
#pragma unroll
        for (int j = 0; j < AH; ++j) F8_READ_FRAG(j, kt_a, vt_a)
    }

#define F8_PIN(x) asm volatile("" ::"v"(x))
#define F8_STEP(I, S_CUR, S_NEXT, EDGE, BAR)                                                                        \
    {                                                                                                               \
        const bool edge = EDGE && (I) == next_edge;                                                                 \
        if (__builtin_expect(edge || vote, 0)) {                                                                    \
            if (edge) {                                                                                             \
                const unsigned live = F8_LIVE(I);                                                                   \
                next_edge = f8_next_edge((I), n0, n01, T);                                                          \
                mask_s(S_CUR, live);                                                                                \
                mx = max_s(S_CUR);                                                                                  \
                _Pragma("unroll") for (int j = 0; j < 8; ++j) {                                                     \
                    const unsigned b4 = (live >> (4 * j)) & 0xF;                                                    \
                    vmask[j] = ((b4 & 1) ? 0xFFu : 0u) | ((b4 & 2) ? 0xFF00u : 0u) | ((b4 & 4) ? 0xFF0000u : 0u) |  \
                               ((b4 & 8) ? 0xFF000000u : 0u);                                                       \
                }                                                                                                   \
            }                                                                                                       \
            /* mx: largest accumulator value, the raw score (LOGLIN) or the score - mref + SHIFT */                  \
            const float delta = fmaxf(fmaxf(mx, __shfl_xor(mx, 32)) - (LOGLIN ? mref : F8_SHIFT), 0.f);             \
            const float alpha = __builtin_amdgcn_exp2f(-delta);                                                     \
            mref += delta;                                                                                          \
            lsum0 *= alpha;                                                                                         \
            lsum1 *= alpha;                                                                                         \
            _Pragma("unroll") for (int db = 0; db < DB; ++db)                                                       \
                _Pragma("unroll") for (int r = 0; r < 16; ++r) st.o[db][r] *= alpha;                                \
            if (LOGLIN) {                                                                                           \
                bias -= 8.0f * delta;                                                                               \
                _Pragma("unroll") for (int r = 0; r < 16; ++r) lacc[r] *= alpha;                                    \
            } else {                                                                                                \
                _Pragma("unroll") for (int r = 0; r < 16; ++r) {                                                    \
                    negm[r] -= delta;                                                                               \
                    S_CUR[0][r] -= delta;                                                                           \
                    S_CUR[1][r] -= delta;                                                                           \
                }                                                                                                   \
            }                                                                                                       \
        }                                                                                                           \
        const unsigned kt_a = lds_a + (((I) + 1) & (NS - 1)) * STAGE_BYTES;            /* K8 of kblock I + 1 */      \
        const unsigned vt_a = lds_a + ((I) & (NS - 1)) * STAGE_BYTES + KB_BYTES;       /* V8 of kblock I     */      \
        const unsigned kn_a = lds_a + (((I) + 2) & (NS - 1)) * STAGE_BYTES;            /* K8 of kblock I + 2 */      \
        i32x8 pb;                                                                                                   \
        float m_run = -INFINITY;                                                                                    \
        _Pragma("unroll") for (int k = 0; k < NSLOT; ++k) {                                                         \
            if (k == 0) __builtin_amdgcn_s_setprio(1);                                                              \
            if (k == NK) __builtin_amdgcn_s_setprio(0);                                                             \
            f8_lds_wait<Plan::wait()>(fr[Plan::buffer(k)][0], fr[Plan::buffer(k)][1]);                                                             \
            if (k < NK) {                                                                                           \
                const int R = k / DH, dh = k % DH;                                                                  \
                S_NEXT[R] = f8_mfma(f8_join(fr[Plan::buffer(k)][0], fr[Plan::buffer(k)][1]), qf[dh],                \
                                    dh == 0 ? (LOGLIN ? zero16 : negm) : S_NEXT[R]);                                \
            } else {                                                                                                \
                const int db = k - NK;                                                                              \
                if (EDGE && edge) {                                                                                 \
                    _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                                 \
                        fr[Plan::buffer(k)][0][j] &= vmask[j];                                                                \
                        fr[Plan::buffer(k)][1][j] &= vmask[4 + j];                                                            \
                    }                                                                                               \
                }                                                                                                   \
                st.o[db] = f8_mfma(f8_join(fr[Plan::buffer(k)][0], fr[Plan::buffer(k)][1]), pb, st.o[db]);          \
                if (LOGLIN && k == NK) lacc = f8_mfma(ones, pb, lacc);     /* row sums of the 8-bit weights */       \
            }                                                                                                       \
            if (k >= DMA_FIRST && (k - DMA_FIRST) % DMA_STEP == 0 && (k - DMA_FIRST) / DMA_STEP < LPW) {            \
                const int v = min((I) + PF, ve - 1);                                                                \
                issue_load(F8_PHYS_KB(v), ((I) + PF) & (NS - 1), (k - DMA_FIRST) / DMA_STEP);                       \
            }                                                                                                       \
            /* the fragment of the slot after next (the first two slots of the next step read kblock I + 2) */      \
            if (k + AH < NSLOT) F8_READ_FRAG(k + AH, kt_a, vt_a)                                                    \
            else F8_READ_FRAG(k + AH - NSLOT, kn_a, vt_a)                                                           \
            if (k < NK) {                                                                                           \
                _Pragma("unroll") for (int g = k * QPS; g < (k + 1) * QPS; ++g) {                                   \
                    const int R = g / 4, r = 4 * (g % 4);                                                           \
                    if (LOGLIN) {                                                                                   \
                        unsigned w = 0;                                                                             \
                        w = __builtin_amdgcn_cvt_pk_u8_f32(__builtin_fmaf(S_CUR[R][r], 8.0f, bias), 0, w);          \
                        w = __builtin_amdgcn_cvt_pk_u8_f32(__builtin_fmaf(S_CUR[R][r + 1], 8.0f, bias), 1, w);      \
                        w = __builtin_amdgcn_cvt_pk_u8_f32(__builtin_fmaf(S_CUR[R][r + 2], 8.0f, bias), 2, w);      \
                        w = __builtin_amdgcn_cvt_pk_u8_f32(__builtin_fmaf(S_CUR[R][r + 3], 8.0f, bias), 3, w);      \
                        pb[g] = int(w);                                                                             \
                        F8_PIN(w);                                                                                  \
                    } else {                                                                                        \
                        const float e0 = __builtin_amdgcn_exp2f(S_CUR[R][r]), e1 = __builtin_amdgcn_exp2f(S_CUR[R][r + 1]);     \
                        const float e2 = __builtin_amdgcn_exp2f(S_CUR[R][r + 2]), e3 = __builtin_amdgcn_exp2f(S_CUR[R][r + 3]); \
                        lsum0 += e0;                                                                                \
                        lsum1 += e1;                                                                                \
                        lsum0 += e2;                                                                                \
                        lsum1 += e3;                                                                                \
                        int w = __builtin_amdgcn_cvt_pk_fp8_f32(e0, e1, 0, false);                                  \
                        w = __builtin_amdgcn_cvt_pk_fp8_f32(e2, e3, w, true);                                       \
                        pb[g] = w;                                                                                  \
                        F8_PIN(w);                                                                                  \
                        F8_PIN(lsum0);                                                                              \
                        F8_PIN(lsum1);                                                                              \
                    }                                                                                               \
                }                                                                                                   \
            } else {                                                                                                \
                _Pragma("unroll") for (int b = (k - NK) * MPS; b < (k - NK + 1) * MPS; b += 2)                      \
                    m_run = fmaxf(fmaxf(m_run, S_NEXT[b >> 4][b & 15]), S_NEXT[b >> 4][(b & 15) + 1]);              \
            }                                                                                                       \
            __builtin_amdgcn_sched_barrier(0);                                                                      \
        }                                                                                                           \
        mx = m_run;                                                                                                 \
        vote = __any(mx - (LOGLIN ? mref : F8_SHIFT) > F8_SLACK);                                                   \
        if (EDGE && edge) {                                                                                         \
            _Pragma("unroll") for (int j = 0; j < 8; ++j) vmask[j] = 0xFFFFFFFFu;                                   \
        }                                                                                                           \
        if (BAR == 1 || (BAR == 2 && RingPlan::barrier_after((I) - vb))) {                                          \
            f8_wait_vmcnt<(PF - LAND) * LPW>();                                                                     \
            __builtin_amdgcn_s_barrier();                                                                           \
        }                                                                                                           \
    }

    int next_edge = f8_next_edge(vb - 1, n0, n01, T);
    bool vote = false;
    int i = vb;
    while (i < ve) {
        while (i < ve && (((i - vb) & 1) || i + 1 >= ve || i == next_edge || i + 1 == next_edge)) {
            F8_STEP(i, sA, sB, 1, 2)
#pragma unroll
            for (int R = 0; R < 2; ++R) sA[R] = sB[R];
            ++i;
        }
        for (int n = (min(ve, next_edge) - i) >> 1; n > 0; --n) {
            F8_STEP(i, sA, sB, 0, 0)
            F8_STEP(i + 1, sB, sA, 0, 1)
            i += 2;
        }
    }
#undef F8_STEP
#undef F8_PIN
#undef F8_READ_FRAG
#undef F8_PHYS_KB
#undef F8_LIVE
    __builtin_amdgcn_s_waitcnt(0);
    // LOGLIN: the MFMA has summed over both key halves already, and both lanes of a query hold that sum
    st.l = LOGLIN ? 0.5f * lacc[0] : lsum0 + lsum1;
}

// A wave without queries in a chunk's short last tile: its share of the loads, waits and barriers only.
template <int D>
__device__ __forceinline__ void f8_segment_loads_only(const AttnParams& p, const AttnChunk& ch, int head, char* lds) {
    constexpr int KB_BYTES = KBLOCK8 * D, STAGE_BYTES = 2 * KB_BYTES;
    constexpr int NF = STAGE_BYTES / 1024;
    constexpr int NS = RingPlan::STAGES, NW = 8, LPW = NF / NW, PF = RingPlan::AHEAD, LAND = RingPlan::LANDED;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n_ranges = ch.n_ranges;
    const int rs0 = ch.rs[0], re0 = ch.re[0];
    int rs1 = ch.rs[1], re1 = ch.re[1], rs2 = ch.rs[2], re2 = ch.re[2];
    if (n_ranges < 2) rs1 = re1 = 0;
    if (n_ranges < 3) rs2 = re2 = 0;
    const int kb0 = rs0 / KBLOCK8, ke0 = (re0 + KBLOCK8 - 1) / KBLOCK8;
    const int kb1 = rs1 / KBLOCK8, ke1 = (re1 + KBLOCK8 - 1) / KBLOCK8;
    const int kb2 = rs2 / KBLOCK8, ke2 = (re2 + KBLOCK8 - 1) / KBLOCK8;
    const int n0 = ke0 - kb0, n01 = n0 + (ke1 - kb1);
    const int vb = 0, ve = n01 + (ke2 - kb2);
    const char* kbase = reinterpret_cast<const char*>(p.k8_cache + head * p.head_stride);
    const char* vbase = reinterpret_cast<const char*>(p.v8_cache + head * p.head_stride);
    const unsigned lane_off = lane * 16;
    auto issue_loads = [&](int v, int stage) {
        const int kb = v + f8_pick(v, n0, n01, kb0, kb1 - n0, kb2 - n01);
        const int64_t kb_off = int64_t(kb) * KB_BYTES;
#pragma unroll
        for (int l = 0; l < LPW; ++l) {
            const int f = wave + NW * l;
            const char* src = (f < NF / 2 ? kbase + f * 1024 : vbase + (f - NF / 2) * 1024) + kb_off + lane_off;
            char* dst = lds + stage * STAGE_BYTES + f * 1024;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src),
                                             (__attribute__((address_space(3))) void*)(dst), 16, 0, 0);
        }
    };
#pragma unroll
    for (int j = 0; j < PF; ++j) issue_loads(min(vb + j, ve - 1), (vb + j) & (NS - 1));
    f8_wait_vmcnt<(PF - LAND) * LPW>();
    __builtin_amdgcn_s_barrier();
    for (int i = vb; i < ve; ++i) {
        issue_loads(min(i + PF, ve - 1), (i + PF) & (NS - 1));
        if (RingPlan::barrier_after(i - vb)) {
            f8_wait_vmcnt<(PF - LAND) * LPW>();
            __builtin_amdgcn_s_barrier();
        }
    }
    __builtin_amdgcn_s_waitcnt(0);
}

// out[row][head][32*db + 8*g + 4*half + i] = O^T register 4*g + i, times 2^v_exp, divided by the row sum
template <int D>
__device__ __forceinline__ void f8_store_out(const AttnParams& p, int head, int q0, int q_end, const F8State<D>& st) {
    constexpr int DB = D / 32;
    const int lane = threadIdx.x & 63, col = lane & 31, half = lane >> 5;
    const float l = st.l + __shfl_xor(st.l, 32);
    const float inv = p.out_scale / l;
    const int row = q0 + col;
    if (row < q_end) {
        uint16_t* dst = p.out + (int64_t(row) * p.H + head) * D + half * 4;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                u32x2 w = {f8_pack_bf16(st.o[db][4 * g] * inv, st.o[db][4 * g + 1] * inv),
                           f8_pack_bf16(st.o[db][4 * g + 2] * inv, st.o[db][4 * g + 3] * inv)};
                *reinterpret_cast<u32x2*>(dst + db * 32 + g * 8) = w;
            }
    }
}

// ---- one workgroup per (head, query tile); placement on the XCDs as in attn_stream.hip
// MODE 0: compiler-scheduled form, 1: explicit pipeline with exact exponentials, 2: explicit pipeline with the
// log-linear weights
template <int D, int MODE>
__global__ __launch_bounds__(F8_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2))) void ll_attn_fp8_kernel(const AttnParams p) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
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
    if (head < 0) return;
    int ci = 0;
    while (ci + 1 < p.n_chunks && tile >= p.chunk[ci + 1].tile_begin) ++ci;
    const AttnChunk& ch = p.chunk[ci];
    const int row_block = ((wave & 3) << 1) | (wave >> 2);        // waves w and w + 4 share a SIMD
    const int q0 = ch.q_begin + (tile - ch.tile_begin) * 256 + row_block * 32;
    if (q0 >= ch.q_end) {
        f8_segment_loads_only<D>(p, ch, head, lds);
        return;
    }
    F8State<D> st;
    if (MODE == 2) f8_segment_sp<D, true>(p, ch, head, q0, lds, st);
    else if (MODE == 1) f8_segment_sp<D, false>(p, ch, head, q0, lds, st);
    else f8_segment<D>(p, ch, head, q0, lds, st);
    f8_store_out<D>(p, head, q0, ch.q_end, st);
}

const AttnVariant kFp8Variants[] = {
    {"d128_fp8", 128, 256, 8 * 2 * KBLOCK8 * 128, ll_attn_fp8_kernel<128, 1>, F8_THREADS, KBLOCK8},
    {"d64_fp8", 64, 256, 8 * 2 * KBLOCK8 * 64, ll_attn_fp8_kernel<64, 1>, F8_THREADS, KBLOCK8},
    {"d128_fp8_simple", 128, 256, 8 * 2 * KBLOCK8 * 128, ll_attn_fp8_kernel<128, 0>, F8_THREADS, KBLOCK8},
    {"d64_fp8_simple", 64, 256, 8 * 2 * KBLOCK8 * 64, ll_attn_fp8_kernel<64, 0>, F8_THREADS, KBLOCK8},
    {"d128_fp8_loglin", 128, 256, 8 * 2 * KBLOCK8 * 128, ll_attn_fp8_kernel<128, 2>, F8_THREADS, KBLOCK8},
    {"d64_fp8_loglin", 64, 256, 8 * 2 * KBLOCK8 * 64, ll_attn_fp8_kernel<64, 2>, F8_THREADS, KBLOCK8},
};
const int kNumFp8Variants = sizeof(kFp8Variants) / sizeof(kFp8Variants[0]);

}  // namespace ll

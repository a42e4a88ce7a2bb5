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
#include <type_traits>

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

template <int D, int PF, int QR>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2))) void ll_attn_sp_kernel(const AttnParams p) {
    constexpr int KS = D / 16;                  // k-steps of S^T = K Q^T, also fragments per K kblock
    constexpr int DB = D / 32;                  // 32-row blocks of O^T
    constexpr int KB_BYTES = KBLOCK * D * 2;
    constexpr int STAGE_BYTES = 2 * KB_BYTES;   // [K kblock | V kblock]
    constexpr int NS = 8;                       // ring stages (a power of two: stage = kblock & 7)
    constexpr int NF = 2 * KS;                  // 1 KB fragments per stage
    constexpr int LPW = NF / 8;                 // loads per wave per kblock
    constexpr int QT = 256;
    static_assert(NF % 8 == 0, "fragments must split over 8 waves");
    static_assert(PF >= 3, "kblock i + 2 must have landed when iteration i starts");
    static_assert(PF + 2 <= NS, "a stage is rewritten two barriers after its last read");
    // QR of the KS query fragments stay in registers, the others live in LDS behind the ring and are
    // read again for every kblock (registers are the scarcer resource: 256 per wave at two waves per SIMD)
    constexpr int QL = KS - QR;
    constexpr int Q_LDS_OFF = NS * STAGE_BYTES;
    static_assert(QR >= 0 && QR <= KS, "QR out of range");

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

    // Q^T fragments (pre-scaled by log2(e)/sqrt(D)): fragment ks holds features 16*ks + 8*half + 0..7
    bf16x8 qf[QR > 0 ? QR : 1];
    char* const q_lds = lds + Q_LDS_OFF + wave * (QL * 1024) + lane * 16;     // this wave's private area
    {
        const int row = min(q0 + col, q_end - 1);
        const uint16_t* src = p.q + (int64_t(row) * p.H + head) * D + half * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const bf16x8 f = *reinterpret_cast<const bf16x8*>(src + ks * 16);
            if (ks < QR) qf[ks] = f;
            else *reinterpret_cast<bf16x8*>(q_lds + (ks - QR) * 1024) = f;
        }
    }
    auto q_frag = [&](int ks) -> bf16x8 {
        if (ks < QR) return qf[ks];
        return *reinterpret_cast<const bf16x8*>(q_lds + (ks - QR) * 1024);
    };

    const char* kbase = reinterpret_cast<const char*>(p.k_cache + head * p.head_stride);
    const char* vbase = reinterpret_cast<const char*>(p.v_cache + head * p.head_stride);

    const int n0 = ke0 - kb0, n01 = n0 + (ke1 - kb1);                     // kblocks in range 0, in ranges 0 and 1
    // physical kblock of virtual kblock v, its range, and whether it is the first or last kblock of a
    // range (only those can be cut by a range boundary; they take the slow path)
#define SP_PHYS_KB(v) ((v) + sp_pick((v), n0, n01, kb0, kb1 - n0, kb2 - n01))
#define SP_LIVE(v) sp_live_mask(SP_PHYS_KB(v) * KBLOCK, sp_pick((v), n0, n01, rs0, rs1, rs2), sp_pick((v), n0, n01, re0, re1, re2), half)

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
    float mref;                                  // reference maximum of this lane's query (log2 domain)
    f32x16 sA, sB;                               // scores minus the reference (log2 domain) of kblocks i and i + 1
    bf16x8 kfr[KS];                              // K fragments of kblock i + 1
    u32x4 vfr[2][DB];                            // V^T fragments of kblock i
    float mx = -INFINITY;                        // largest score of kblock i among this lane's keys (kblock 0: reference already exact)

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

    // ---- prologue: scores of kblock 0 against a zero reference, then the true first reference
    read_k(0, kfr);
#pragma unroll
    for (int r = 0; r < 16; ++r) sA[r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) sA = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr[ks], q_frag(ks), sA, 0, 0, 0);
    mask_s(sA, SP_LIVE(0));
    {
        const float m = max_s(sA);
        const float m0 = fmaxf(m, __shfl_xor(m, 32));     // a kblock of a range holds a live key: finite
        mref = m0;
    }
    read_k(1 % NS, kfr);

    // One kblock per step.  S_CUR holds the scores of kblock I on entry, S_NEXT those of kblock I + 1 on exit;
    // the loop below alternates the two register sets so that no copy is needed.
    //
    // A step is NSLOT = KS + 2*DB slots, each opened by one MFMA: first the KS MFMAs of S^T = K Q^T for kblock
    // I+1, then the 2*DB MFMAs of O^T += V^T P^T for kblock I.  The vector work of kblock I rides in their shadow
    // as a skewed pipeline over the 8 score pairs of a lane, so that no instruction waits for the one before it:
    //     slot w-1: subtract the reference from pair w      slot w+1: pack pair w to bf16 (one P^T word)
    //     slot w  : exp2 of pair w                          slot w+2: add the packed pair to the row sum
    // the last slots take the running maximum of the new scores, and every slot reads one fragment for later:
    // V^T of kblock I during the first KS slots, K of kblock I+2 afterwards.  A scheduling fence after every
    // slot keeps the compiler from regrouping the instructions and the empty asm statements pin each stage's
    // results inside its slot.  Before the slots: the rare path (a score above the reference by more than the
    // slack, or a kblock that may be cut by a range boundary: mask, move the reference, rescale O and the sums).
    // After them: the wave waits for its own older loads and the workgroup barrier hands the ring stages over.
    constexpr int NSLOT = KS + 2 * DB;
    constexpr int MAX_FIRST = NSLOT - 4;         // slots that take the maximum (the S^T chain has drained by then)
    // slot of each stage of score pair w; the packed pair must exist before the MFMA that consumes it
    auto slot_cvt = [](int w) { const int dl = KS + (w >> 2) * DB - 1; return w + 1 < dl ? w + 1 : dl; };
    auto slot_exp = [slot_cvt](int w) { return w < slot_cvt(w) ? w : slot_cvt(w); };
    auto slot_sub = [slot_exp](int w) { const int a = w > 0 ? w - 1 : 0; return a < slot_exp(w) ? a : slot_exp(w); };
    auto slot_sum = [](int w) { return w + 2 < NSLOT - 1 ? w + 2 : NSLOT - 1; };
#define SP_PIN(x) asm volatile("" ::"v"(x))
#define SP_STEP(I, S_CUR, S_NEXT)                                                                                  \
    {                                                                                                               \
        const bool edge = (I) == next_edge;                                                                         \
        if (edge || __any(mx > thr)) {                                                                              \
            if (edge) {                                                                                             \
                mask_s(S_CUR, SP_LIVE(I));                                                                          \
                mx = max_s(S_CUR);                                                                                  \
                next_edge = sp_next_edge((I), n0, n01, T);                                                          \
            }                                                                                                       \
            const float mnew = fmaxf(fmaxf(mx, __shfl_xor(mx, 32)), mref);                                          \
            const float alpha = __builtin_amdgcn_exp2f(mref - mnew);                                                \
            mref = mnew;                                                                                            \
            thr = mnew + SP_RESCALE_SLACK;                                                                          \
            lsum0 *= alpha;                                                                                         \
            lsum1 *= alpha;                                                                                         \
            _Pragma("unroll") for (int db = 0; db < DB; ++db)                                                       \
                _Pragma("unroll") for (int r = 0; r < 16; ++r) o[db][r] *= alpha;                                   \
        }                                                                                                           \
        const char* vt = lds + (((I)) & (NS - 1)) * STAGE_BYTES + KB_BYTES + lane_off;                              \
        const char* kt = lds + (((I) + 2) & (NS - 1)) * STAGE_BYTES + lane_off;                                     \
        float d0[8], d1[8];                                                                                         \
        unsigned pb[2][4];                                                                                          \
        float m_run = -INFINITY;                                                                                    \
        _Pragma("unroll") for (int r = 0; r < 16; ++r) S_NEXT[r] = 0.f;                                             \
        _Pragma("unroll") for (int k = 0; k < NSLOT; ++k) {                                                         \
            if (k < KS) {                                                                                           \
                S_NEXT = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr[k], q_frag(k), S_NEXT, 0, 0, 0);               \
            } else {                                                                                                \
                const int t = (k - KS) / DB, db = (k - KS) % DB;                                                    \
                const u32x4 bv = {pb[t][0], pb[t][1], pb[t][2], pb[t][3]};                                          \
                o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vfr[t][db]),             \
                                                                 __builtin_bit_cast(bf16x8, bv), o[db], 0, 0, 0);   \
            }                                                                                                       \
            if (k == 0) {                                                                                           \
                const int v = min((I) + PF, T - 1);                                                                 \
                issue_loads(SP_PHYS_KB(v), ((I) + PF) & (NS - 1));                                                  \
            }                                                                                                       \
            _Pragma("unroll") for (int w = 0; w < 8; ++w) {                                                         \
                if (k == slot_sub(w)) {                                                                             \
                    d0[w] = S_CUR[2 * w] - mref;                                                                    \
                    d1[w] = S_CUR[2 * w + 1] - mref;                                                                \
                    SP_PIN(d0[w]);                                                                                  \
                    SP_PIN(d1[w]);                                                                                  \
                }                                                                                                   \
                if (k == slot_exp(w)) {                                                                             \
                    d0[w] = __builtin_amdgcn_exp2f(d0[w]);                                                          \
                    d1[w] = __builtin_amdgcn_exp2f(d1[w]);                                                          \
                    SP_PIN(d0[w]);                                                                                  \
                    SP_PIN(d1[w]);                                                                                  \
                }                                                                                                   \
                if (k == slot_cvt(w)) {                                                                             \
                    pb[w >> 2][w & 3] = sp_pack_bf16(d0[w], d1[w]);                                                 \
                    SP_PIN(pb[w >> 2][w & 3]);                                                                      \
                }                                                                                                   \
                if (k == slot_sum(w)) {                                                                             \
                    if (w < 4) lsum0 = sp_pair_sum(pb[w >> 2][w & 3], lsum0);                                       \
                    else lsum1 = sp_pair_sum(pb[w >> 2][w & 3], lsum1);                                             \
                }                                                                                                   \
            }                                                                                                       \
            if (k >= MAX_FIRST) {                                                                                   \
                const int r = (k - MAX_FIRST) * 4;                                                                  \
                m_run = fmaxf(fmaxf(m_run, S_NEXT[r]), S_NEXT[r + 1]);                                              \
                m_run = fmaxf(fmaxf(m_run, S_NEXT[r + 2]), S_NEXT[r + 3]);                                          \
            }                                                                                                       \
            if (k < KS) {                                                                                           \
                _Pragma("unroll") for (int f = k * 2 * DB / KS; f < (k + 1) * 2 * DB / KS; ++f)                     \
                    vfr[f / DB][f % DB] = *reinterpret_cast<const u32x4*>(vt + ((f % DB) * 2 + f / DB) * 1024);     \
            } else {                                                                                                \
                _Pragma("unroll") for (int f = (k - KS) * KS / (2 * DB); f < (k - KS + 1) * KS / (2 * DB); ++f)     \
                    kfr[f] = *reinterpret_cast<const bf16x8*>(kt + f * 1024);                                       \
            }                                                                                                       \
            __builtin_amdgcn_sched_barrier(0);                                                                      \
            if (k == KS - 1 && edge) mask_v(vfr, SP_LIVE(I));                                                       \
        }                                                                                                           \
        mx = m_run;                                                                                                 \
        sp_wait_vmcnt<(PF - 3) * LPW>();                                                                            \
        __builtin_amdgcn_s_barrier();                                                                               \
    }

    int next_edge = 0;                           // next kblock that may be cut by a range boundary
    float thr = mref + SP_RESCALE_SLACK;         // a score above this moves the reference
    for (int i = 0; i < T; i += 2) {
        SP_STEP(i, sA, sB)
        if (i + 1 >= T) break;
        SP_STEP(i + 1, sB, sA)
    }
#undef SP_STEP
#undef SP_PIN
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

#define SP_VARIANT(D, PF, QR)                                                                         \
    { "d" #D "_sp_pf" #PF "_qr" #QR, D, 256, 8 * 2 * KBLOCK * D * 2 + (D / 16 - QR) * 8 * 1024,         \
      ll_attn_sp_kernel<D, PF, QR>, 512 }
const AttnVariant kStreamVariants[] = {
    SP_VARIANT(128, 4, 8),
    SP_VARIANT(128, 6, 8),
    SP_VARIANT(64, 4, 4),
};
const int kNumStreamVariants = sizeof(kStreamVariants) / sizeof(kStreamVariants[0]);

}  // namespace ll

// Backward pass of the train-time rule (paper Sec. 3.2 and Sec. 3.3 "Consistency between Training and Inference"):
// gradients of the clip's attention (sink + detached window + the clip itself, chunk by chunk) with respect to the
// clip's own rotated queries, rotated keys and values.
//
// With P = softmax over a query's key set (kept as lse, the log2 of the row sum, by the forward kernel),
//     dV_j = sum_i P_ij dO_i,   dP_ij = dO_i . V_j,   dZ_ij = P_ij (dP_ij - delta_i),   delta_i = dO_i . O_i,
//     Gq_i = sum_j dZ_ij K'_j,  Gk_j = sum_i dZ_ij q'_i
// (the factors 1/sqrt(D) and ln 2 and the turn back through the rotary embedding follow in ll_bwd_finish_kernel).
// Two kernels, both in the forward kernel's formulation: a wave owns 32 columns (queries, or keys), every lane one
// column, and the other side streams past in blocks of 32 rows as ready-made MFMA fragments (kernels.h): products
// that contract over the feature axis take "K-style" fragments as the A operand and the column's own row as B;
// products that contract over the streamed rows take "V^T-style" fragments as A and the accumulator registers of the
// step before (P or dZ, rounded to bf16) as B, with no movement between lanes.
//   ll_bwd_dq_kernel:  columns = queries;  streams K' (K-style), V (K-style), K'^T (V^T-style);   Gq^T += K'^T dZ^T
//   ll_bwd_dkv_kernel: columns = clip keys; streams q', dO (K-style), dO^T, q'^T (V^T-style);
//                      dV^T += dO^T P,  Gk^T += q'^T dZ
// The streamed blocks reach LDS by direct loads into a ring of stages, two blocks ahead; one workgroup of 8 waves
// (4 at head_dim 64) per 256 (128) columns.
#include "kernels.h"

namespace ll {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

__device__ inline unsigned bw_pack_bf16(float a, float b) {
    f32x2 v = {a, b};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2));
}

// Dead rows (outside the streamed range, in the blocks at its ends) get weight exactly zero: score -inf, so that
// P = 2^(-inf - lse) = 0 and dZ = 0 * (0 - delta) = 0.  The fragments they multiply are not cleared: every resident
// frame of a step holds finite values written by this step, so 0 * fragment = 0.  (The inference kernels do clear
// them, since a ring slot outside the key set may hold anything.)
__device__ inline void bw_kill_dead_rows(f32x16& s, f32x16& dp, int row0, int lo, int hi, int half) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int row = row0 + 16 * (r >> 3) + 8 * half + (r & 7);      // the row register r stands for
        if (row < lo || row >= hi) {
            s[r] = -INFINITY;
            dp[r] = 0.f;
        }
    }
}

// s_waitcnt that only waits for vector-memory loads: at most N outstanding.
template <int N>
__device__ __forceinline__ void bw_wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (0x7 << 4) | (0xF << 8));
}

// Barrier without the fence of __syncthreads (which would wait for every outstanding load, the prefetched blocks
// included); the "memory" clobber keeps the compiler from moving LDS reads across it.
__device__ __forceinline__ void bw_barrier() { asm volatile("s_barrier" ::: "memory"); }

// Walks the 32-row blocks of a group's streamed ranges in order; past the end it stays on the last block.  The ranges
// are copied into registers once (no kernel-argument loads inside the loop).
struct BwRanges { int n, rs0, re0, rs1, re1; };
__device__ inline BwRanges bw_ranges(const BwdGroup& g) {
    BwRanges r{g.n_ranges, g.rs[0], g.re[0], g.rs[1], g.re[1]};
    if (r.n < 2) r.rs1 = r.re1 = 0;
    return r;
}
struct BwIter { int rng, kb, kb_end; };
__device__ inline void bw_iter_init(const BwRanges& g, BwIter& it) {
    it.rng = 0;
    it.kb = g.rs0 / KBLOCK;
    it.kb_end = (g.re0 + KBLOCK - 1) / KBLOCK;
}
__device__ inline void bw_iter_advance(const BwRanges& g, BwIter& it) {
    if (it.kb + 1 < it.kb_end) {
        ++it.kb;
    } else if (it.rng + 1 < g.n) {
        it.rng = 1;
        it.kb = g.rs1 / KBLOCK;
        it.kb_end = (g.re1 + KBLOCK - 1) / KBLOCK;
    }
}

// The streamed blocks go from memory straight into a ring of LDS stages (global_load_lds, one 1 KB fragment per wave
// and load), PF blocks ahead of the block being worked on.  Per block: issue the loads of block it + PF, wait until
// this wave's loads of block it have landed (all but the PF * LPW youngest), barrier (every wave's have), compute.
// A wave can be one block ahead of the slowest one, so the stage it writes, (it + 1 + PF) mod NS, must differ from the
// one still being read, it mod NS: NS = PF + 2.
constexpr int BW_PF = 2, BW_NS = 4;

// Workgroup -> (head, column tile): contiguous runs of items per XCD, as in the forward kernels.
__device__ inline bool bw_item(int n_tiles, int H, int& head, int& tile) {
    const int total = n_tiles * H;
    const int per_xcd = (total + 7) >> 3;
    const int item = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if ((int)(blockIdx.x >> 3) >= per_xcd || item >= total) return false;
    head = item / n_tiles;
    tile = item % n_tiles;
    return true;
}

// The B operand of a feature-contracting product for the column at token `slot` of a K-style region: fragment ks is
// features 16 ks + 8 half + 0..7 of that row.
template <int D>
__device__ inline void bw_load_kstyle_row(const uint16_t* region, int64_t slot, int half, bf16x8 (&f)[D / 16]) {
    const uint16_t* base = region + (slot / KBLOCK) * (KBLOCK * D) + swap23(int(slot % KBLOCK)) * 8;
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) f[ks] = *reinterpret_cast<const bf16x8*>(base + (2 * ks + half) * (32 * 8));
}

// ---------------------------------------------------------------------------------------------------------------
template <int D, int NW>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(2, 2))) void ll_bwd_dq_kernel(const BwdParams p) {
    constexpr int KS = D / 16, DB = D / 32;
    constexpr int KB_BYTES = KBLOCK * D * 2;
    constexpr int NREG = 3;                           // streamed regions per block
    extern __shared__ __attribute__((aligned(16))) char lds[];   // [BW_NS][NREG][KB_BYTES]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, half = lane >> 5;
    int head, tile;
    if (!bw_item(p.n_tiles, p.H, head, tile)) return;
    int gi = 0;
    while (gi + 1 < p.n_groups && tile >= p.group[gi + 1].tile_begin) ++gi;
    const BwdGroup& g = p.group[gi];
    const int q0 = g.c_begin + (tile - g.tile_begin) * (NW * 32) + wave * 32;
    const int row = min(q0 + col, g.c_end - 1);

    bf16x8 qf[KS], dof[KS];
    {
        const int64_t off = (int64_t(row) * p.H + head) * D + half * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            qf[ks] = *reinterpret_cast<const bf16x8*>(p.q + off + ks * 16);
            dof[ks] = *reinterpret_cast<const bf16x8*>(p.dout + off + ks * 16);
        }
    }
    const float lse = p.lse[int64_t(head) * p.row_stride + row];
    const float delta = p.delta[int64_t(head) * p.row_stride + row];

    f32x16 acc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[db][r] = 0.f;

    const char* src[NREG] = {reinterpret_cast<const char*>(p.s_k1 + head * p.hs_k1),
                             reinterpret_cast<const char*>(p.s_k2 + head * p.hs_k2),
                             reinterpret_cast<const char*>(p.s_t1 + head * p.hs_t1)};

    int n_blocks = 0;
    for (int r = 0; r < g.n_ranges; ++r) n_blocks += (g.re[r] + KBLOCK - 1) / KBLOCK - g.rs[r] / KBLOCK;

    constexpr int FPR = KB_BYTES / 1024;              // 1 KB fragments per region and block
    constexpr int LPW = NREG * FPR / NW;              // loads per wave and block
    static_assert((NREG * FPR) % NW == 0, "fragments must split over the waves");
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    auto issue = [&](int kblk, int stage) {
#pragma unroll
        for (int l = 0; l < LPW; ++l) {
            const int f = wave_u + NW * l, region = f / FPR, fr = f % FPR;      // wave-uniform
            const char* from = src[region] + int64_t(kblk) * KB_BYTES + fr * 1024 + lane * 16;
            char* to = lds + (stage * NREG + region) * KB_BYTES + fr * 1024;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(from),
                                             (__attribute__((address_space(3))) void*)(to), 16, 0, 0);
        }
    };
    const BwRanges gr = bw_ranges(g);
    BwIter li, ci;
    bw_iter_init(gr, li);
    bw_iter_init(gr, ci);
#pragma unroll
    for (int j = 0; j < BW_PF; ++j) {
        issue(li.kb, j);
        bw_iter_advance(gr, li);
    }
    // Software pipeline: the two feature-contracting products of block it + 1 are issued before the vector work of
    // block it (exp2, dZ, packing), which does not depend on them, so the matrix pipe runs under that work.
    auto scores = [&](const char* blk, f32x16& s, f32x16& dp) {
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = dp[r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const bf16x8 ak = *reinterpret_cast<const bf16x8*>(blk + ks * 1024 + lane * 16);
            const bf16x8 av = *reinterpret_cast<const bf16x8*>(blk + KB_BYTES + ks * 1024 + lane * 16);
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ak, qf[ks], s, 0, 0, 0);
            dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, dof[ks], dp, 0, 0, 0);
        }
    };
    // One block: the vector work and the row-contracting product of block `it` from its scores (s, dp), and the scores
    // of block it + 1 (past the end: the last block again, unused) into (s_next, dp_next).
    auto block = [&](int it, f32x16& s, f32x16& dp, f32x16& s_next, f32x16& dp_next) {
        issue(li.kb, (it + BW_PF) & (BW_NS - 1));
        bw_iter_advance(gr, li);
        bw_wait_vmcnt<(BW_PF - 1) * LPW>();          // this wave's loads of block it + 1 have landed
        bw_barrier();

        const char* blk = lds + (it & (BW_NS - 1)) * NREG * KB_BYTES;
        const int key0 = ci.kb * KBLOCK, cur_rs = ci.rng ? gr.rs1 : gr.rs0, cur_re = ci.rng ? gr.re1 : gr.re0;
        bw_iter_advance(gr, ci);
        if (key0 < cur_rs || key0 + KBLOCK > cur_re)  // uniform: only the blocks at the ends of a range
            bw_kill_dead_rows(s, dp, key0, cur_rs, cur_re, half);

        scores(lds + ((it + 1) & (BW_NS - 1)) * NREG * KB_BYTES, s_next, dp_next);

        unsigned dz[2][4];
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float z[2];
#pragma unroll
                for (int k = 0; k < 2; ++k) {
                    const int r = 8 * t + 2 * e + k;
                    const float pr = __builtin_amdgcn_exp2f(s[r] - lse);
                    z[k] = pr * (dp[r] - delta);
                }
                dz[t][e] = bw_pack_bf16(z[0], z[1]);
            }
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const u32x4 bv = {dz[t][0], dz[t][1], dz[t][2], dz[t][3]};
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                const bf16x8 a = *reinterpret_cast<const bf16x8*>(blk + 2 * KB_BYTES + (db * 2 + t) * 1024 + lane * 16);
                acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, __builtin_bit_cast(bf16x8, bv), acc[db], 0, 0, 0);
            }
        }
    };
    f32x16 s0, dp0, s1, dp1;
    bw_wait_vmcnt<(BW_PF - 1) * LPW>();              // block 0 has landed
    bw_barrier();
    scores(lds, s0, dp0);
    for (int it = 0; it < n_blocks; it += 2) {       // two blocks per trip: the two score sets swap roles, no copies
        block(it, s0, dp0, s1, dp1);
        if (it + 1 < n_blocks) block(it + 1, s1, dp1, s0, dp0);
    }
    bw_wait_vmcnt<0>();                               // the loads issued past the end have landed before the wave leaves

    // Gq[row][head][32 db + 8 g + 4 half + i] = accumulator register 4 g + i
    if (q0 + col < g.c_end) {
        float* dst = p.g1 + (int64_t(q0 + col) * p.H + head) * D + half * 4;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int gg = 0; gg < 4; ++gg) {
                const f32x4 w = {acc[db][4 * gg], acc[db][4 * gg + 1], acc[db][4 * gg + 2], acc[db][4 * gg + 3]};
                *reinterpret_cast<f32x4*>(dst + db * 32 + gg * 8) = w;
            }
    }
}

// ---------------------------------------------------------------------------------------------------------------
template <int D, int NW>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(2, 2))) void ll_bwd_dkv_kernel(const BwdParams p) {
    constexpr int KS = D / 16, DB = D / 32;
    constexpr int KB_BYTES = KBLOCK * D * 2;
    constexpr int NREG = 4;
    extern __shared__ __attribute__((aligned(16))) char lds[];   // [BW_NS][NREG x KB_BYTES | 256]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, half = lane >> 5;
    int head, tile;
    if (!bw_item(p.n_tiles, p.H, head, tile)) return;
    int gi = 0;
    while (gi + 1 < p.n_groups && tile >= p.group[gi + 1].tile_begin) ++gi;
    const BwdGroup& g = p.group[gi];
    const int k0 = g.c_begin + (tile - g.tile_begin) * (NW * 32) + wave * 32;     // clip token index of this wave's first key
    const int key = min(k0 + col, g.c_end - 1);

    // this column's K' and V rows, from the K-style regions of all resident frames (the clip is their tail)
    bf16x8 kf[KS], vf[KS];
    bw_load_kstyle_row<D>(p.c_k1 + head * p.hc_k1, p.col_slot0 + key, half, kf);
    bw_load_kstyle_row<D>(p.c_k2 + head * p.hc_k2, p.col_slot0 + key, half, vf);

    f32x16 acc_v[DB], acc_k[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_v[db][r] = acc_k[db][r] = 0.f;

    const char* src[NREG] = {reinterpret_cast<const char*>(p.s_k1 + head * p.hs_k1),    // q'   K-style
                             reinterpret_cast<const char*>(p.s_k2 + head * p.hs_k2),    // dO   K-style
                             reinterpret_cast<const char*>(p.s_t1 + head * p.hs_t1),    // dO^T V^T-style
                             reinterpret_cast<const char*>(p.s_t2 + head * p.hs_t2)};   // q'^T V^T-style
    const float* lse_h = p.lse + int64_t(head) * p.row_stride;
    const float* delta_h = p.delta + int64_t(head) * p.row_stride;

    const int row_lo = g.rs[0], row_hi = g.re[0];                                 // one range of query rows
    const int qb_begin = row_lo / KBLOCK, qb_end = (row_hi + KBLOCK - 1) / KBLOCK;
    const int n_blocks = qb_end - qb_begin;

    constexpr int FPR = KB_BYTES / 1024;
    constexpr int LPW = NREG * FPR / NW;
    static_assert((NREG * FPR) % NW == 0, "fragments must split over the waves");
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    // A stage holds the block's four fragment regions and, behind them, the 32 lse and 32 delta values of its rows
    // (256 bytes, one dword per lane; every wave loads them, all the same values, so that all waves count the same
    // number of loads).
    constexpr int STAGE_BYTES = NREG * KB_BYTES + 256;
    const float* aux_src = (lane < 32 ? lse_h : delta_h - 32) + lane;
    auto issue = [&](int blk_i, int stage) {
#pragma unroll
        for (int l = 0; l < LPW; ++l) {
            const int f = wave_u + NW * l, region = f / FPR, fr = f % FPR;
            const char* from = src[region] + int64_t(blk_i) * KB_BYTES + fr * 1024 + lane * 16;
            char* to = lds + stage * STAGE_BYTES + region * KB_BYTES + fr * 1024;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(from),
                                             (__attribute__((address_space(3))) void*)(to), 16, 0, 0);
        }
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(aux_src + blk_i * KBLOCK),
                                         (__attribute__((address_space(3))) void*)(lds + stage * STAGE_BYTES + NREG * KB_BYTES), 4, 0, 0);
    };
    constexpr int LOADS = LPW + 1;                    // per wave and block
#pragma unroll
    for (int j = 0; j < BW_PF; ++j) issue(min(qb_begin + j, qb_end - 1), j);

    for (int it = 0; it < n_blocks; ++it) {
        const int qb = qb_begin + it;
        issue(min(qb + BW_PF, qb_end - 1), (it + BW_PF) & (BW_NS - 1));
        bw_wait_vmcnt<BW_PF * LOADS>();
        bw_barrier();

        const char* blk = lds + (it & (BW_NS - 1)) * STAGE_BYTES;
        const int row0 = qb * KBLOCK;

        f32x16 s, dp;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = dp[r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const bf16x8 aq = *reinterpret_cast<const bf16x8*>(blk + ks * 1024 + lane * 16);
            const bf16x8 ad = *reinterpret_cast<const bf16x8*>(blk + KB_BYTES + ks * 1024 + lane * 16);
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aq, kf[ks], s, 0, 0, 0);
            dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ad, vf[ks], dp, 0, 0, 0);
        }
        if (row0 < row_lo || row0 + KBLOCK > row_hi)     // uniform: only the blocks at the ends of the range
            bw_kill_dead_rows(s, dp, row0, row_lo, row_hi, half);
        // register r stands for query row0 + 16(r/8) + 8 half + r%8: its lse and delta come from the stage's last
        // 256 bytes, 8 consecutive values per (t, half) (rows past the clip read the zero padding of the two vectors;
        // they are dead rows)
        unsigned pw[2][4], dz[2][4];
        const float* aux = reinterpret_cast<const float*>(blk + NREG * KB_BYTES);
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int rb = 16 * t + 8 * half;
            const f32x4 l0 = *reinterpret_cast<const f32x4*>(aux + rb), l1 = *reinterpret_cast<const f32x4*>(aux + rb + 4);
            const f32x4 d0 = *reinterpret_cast<const f32x4*>(aux + 32 + rb), d1 = *reinterpret_cast<const f32x4*>(aux + 32 + rb + 4);
            const float lv[8] = {l0[0], l0[1], l0[2], l0[3], l1[0], l1[1], l1[2], l1[3]};
            const float dl[8] = {d0[0], d0[1], d0[2], d0[3], d1[0], d1[1], d1[2], d1[3]};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float pv[2], zv[2];
#pragma unroll
                for (int k = 0; k < 2; ++k) {
                    const int r = 8 * t + 2 * e + k;
                    const float pr = __builtin_amdgcn_exp2f(s[r] - lv[2 * e + k]);
                    pv[k] = pr;
                    zv[k] = pr * (dp[r] - dl[2 * e + k]);
                }
                pw[t][e] = bw_pack_bf16(pv[0], pv[1]);
                dz[t][e] = bw_pack_bf16(zv[0], zv[1]);
            }
        }
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const u32x4 bp = {pw[t][0], pw[t][1], pw[t][2], pw[t][3]};
            const u32x4 bz = {dz[t][0], dz[t][1], dz[t][2], dz[t][3]};
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                const bf16x8 a_d = *reinterpret_cast<const bf16x8*>(blk + 2 * KB_BYTES + (db * 2 + t) * 1024 + lane * 16);
                const bf16x8 a_q = *reinterpret_cast<const bf16x8*>(blk + 3 * KB_BYTES + (db * 2 + t) * 1024 + lane * 16);
                acc_v[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_d, __builtin_bit_cast(bf16x8, bp), acc_v[db], 0, 0, 0);
                acc_k[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_q, __builtin_bit_cast(bf16x8, bz), acc_k[db], 0, 0, 0);
            }
        }
    }
    bw_wait_vmcnt<0>();

    if (k0 + col < g.c_end) {
        const int64_t off = (int64_t(k0 + col) * p.H + head) * D + half * 4;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int gg = 0; gg < 4; ++gg) {
                const f32x4 w = {acc_k[db][4 * gg], acc_k[db][4 * gg + 1], acc_k[db][4 * gg + 2], acc_k[db][4 * gg + 3]};
                *reinterpret_cast<f32x4*>(p.g1 + off + db * 32 + gg * 8) = w;
                const unsigned v0 = bw_pack_bf16(acc_v[db][4 * gg], acc_v[db][4 * gg + 1]);
                const unsigned v1 = bw_pack_bf16(acc_v[db][4 * gg + 2], acc_v[db][4 * gg + 3]);
                typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
                const u32x2 wv = {v0, v1};
                *reinterpret_cast<u32x2*>(p.dv + off + db * 32 + gg * 8) = wv;
            }
    }
}

// ---------------------------------------------------------------------------------------------------------------
// delta[head][row] = sum_d dO[row][head][d] * O[row][head][d], O being the forward's output before its rounding to
// bf16; D / 8 lanes per (row, head), 8 features each.
template <int D>
__global__ __launch_bounds__(256) void ll_bwd_delta_kernel(const float* out, const uint16_t* dout, float* delta,
                                                           int rows, int H, int64_t row_stride) {
    constexpr int LPR = D / 8;                        // lanes per (row, head)
    const int64_t idx = (int64_t(blockIdx.x) * 256 + threadIdx.x) / LPR;   // (row, head) pair
    const int part = threadIdx.x % LPR;
    const bool on = idx < int64_t(rows) * H;
    float acc = 0.f;
    if (on) {
        const f32x4 a0 = *reinterpret_cast<const f32x4*>(out + idx * D + part * 8);
        const f32x4 a1 = *reinterpret_cast<const f32x4*>(out + idx * D + part * 8 + 4);
        const bf16x8 b = *reinterpret_cast<const bf16x8*>(dout + idx * D + part * 8);
#pragma unroll
        for (int e = 0; e < 4; ++e) acc += a0[e] * float(b[e]) + a1[e] * float(b[e + 4]);
    }
#pragma unroll
    for (int m = LPR / 2; m >= 1; m >>= 1) acc += __shfl_xor(acc, m);
    if (on && part == 0) delta[(idx % H) * row_stride + idx / H] = acc;
}

// dq = R^T(Gq) / sqrt(D), dk = R^T(Gk) ln 2: back through the rotary embedding (the rotation by the opposite angle)
// with the factors the two kernels above left out.  One workgroup per (32 tokens of one frame, head).
template <int D>
__global__ __launch_bounds__(256) void ll_bwd_finish_kernel(const BwdFinishParams p) {
    constexpr int CH = D / 8;
    __shared__ float2 t_cs[64];
    const int tid = threadIdx.x, head = blockIdx.y;
    const int segs = (p.P + 31) / 32;
    const int fi = blockIdx.x / segs, seg = blockIdx.x % segs;
    if (tid < p.rope.n_t) {
        double sn, cs;
        sincos(double(p.frame0 + fi) * p.rope.inv_freq_t[tid], &sn, &cs);
        t_cs[tid] = make_float2(float(cs), float(sn));
    }
    __syncthreads();
    const int ntok = min(32, p.P - seg * 32);
    for (int item = tid; item < ntok * CH; item += 256) {
        const int ti = item / CH, c = item % CH;
        const int tok = seg * 32 + ti;
        const int y = tok / p.grid_w, x = tok % p.grid_w;
        const int64_t off = ((int64_t(fi) * p.P + tok) * p.H + head) * D + c * 8;
        const f32x4 q0 = *reinterpret_cast<const f32x4*>(p.gq + off), q1 = *reinterpret_cast<const f32x4*>(p.gq + off + 4);
        const f32x4 k0 = *reinterpret_cast<const f32x4*>(p.gk + off), k1 = *reinterpret_cast<const f32x4*>(p.gk + off + 4);
        const float gq[8] = {q0[0], q0[1], q0[2], q0[3], q1[0], q1[1], q1[2], q1[3]};
        const float gk[8] = {k0[0], k0[1], k0[2], k0[3], k1[0], k1[1], k1[2], k1[3]};
        unsigned qo[4], ko[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int pi = c * 4 + e;
            float2 cs;
            if (pi < p.rope.n_t) cs = t_cs[pi];
            else if (pi < p.rope.n_t + p.rope.n_h) cs = p.rope.row_cs[y * p.rope.n_h + (pi - p.rope.n_t)];
            else cs = p.rope.col_cs[x * p.rope.n_w + (pi - p.rope.n_t - p.rope.n_h)];
            // transpose of (re, im) -> (re cos - im sin, re sin + im cos)
            qo[e] = bw_pack_bf16((gq[2 * e] * cs.x + gq[2 * e + 1] * cs.y) * p.q_mul, (gq[2 * e + 1] * cs.x - gq[2 * e] * cs.y) * p.q_mul);
            ko[e] = bw_pack_bf16((gk[2 * e] * cs.x + gk[2 * e + 1] * cs.y) * p.k_mul, (gk[2 * e + 1] * cs.x - gk[2 * e] * cs.y) * p.k_mul);
        }
        *reinterpret_cast<u32x4*>(p.dq + off) = u32x4{qo[0], qo[1], qo[2], qo[3]};
        *reinterpret_cast<u32x4*>(p.dk + off) = u32x4{ko[0], ko[1], ko[2], ko[3]};
    }
}

// ---------------------------------------------------------------------------------------------------------------
static hipError_t set_lds(const void* fn, int bytes, bool& done) {
    if (done) return hipSuccess;
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess) done = true;
    return e;
}

// Columns per workgroup: 8 waves (one staged block serves 256 columns) where a kblock splits over 512 threads.
int bwd_tile_cols(int D) { return D == 128 ? 256 : 128; }

hipError_t launch_bwd_dq(const BwdParams& p, hipStream_t s) {
    const int total = p.n_tiles * p.H;
    if (total <= 0) return hipSuccess;
    const int grid = ((total + 7) / 8) * 8, lds = BW_NS * 3 * KBLOCK * p.D * 2;
    static bool done128 = false, done64 = false;
    if (p.D == 128) {
        hipError_t e = set_lds(reinterpret_cast<const void*>(ll_bwd_dq_kernel<128, 8>), lds, done128);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((ll_bwd_dq_kernel<128, 8>), dim3(grid), dim3(512), lds, s, p);
    } else if (p.D == 64) {
        hipError_t e = set_lds(reinterpret_cast<const void*>(ll_bwd_dq_kernel<64, 4>), lds, done64);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((ll_bwd_dq_kernel<64, 4>), dim3(grid), dim3(256), lds, s, p);
    } else return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_bwd_dkv(const BwdParams& p, hipStream_t s) {
    const int total = p.n_tiles * p.H;
    if (total <= 0) return hipSuccess;
    const int grid = ((total + 7) / 8) * 8, lds = BW_NS * (4 * KBLOCK * p.D * 2 + 256);
    static bool done128 = false, done64 = false;
    if (p.D == 128) {
        hipError_t e = set_lds(reinterpret_cast<const void*>(ll_bwd_dkv_kernel<128, 8>), lds, done128);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((ll_bwd_dkv_kernel<128, 8>), dim3(grid), dim3(512), lds, s, p);
    } else if (p.D == 64) {
        hipError_t e = set_lds(reinterpret_cast<const void*>(ll_bwd_dkv_kernel<64, 4>), lds, done64);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((ll_bwd_dkv_kernel<64, 4>), dim3(grid), dim3(256), lds, s, p);
    } else return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_bwd_delta(const float* out, const uint16_t* dout, float* delta, int rows, int H, int D,
                            int64_t row_stride, hipStream_t s) {
    if (rows <= 0) return hipSuccess;
    const int64_t threads = int64_t(rows) * H * (D / 8);
    const unsigned grid = unsigned((threads + 255) / 256);
    if (D == 128) hipLaunchKernelGGL(ll_bwd_delta_kernel<128>, dim3(grid), dim3(256), 0, s, out, dout, delta, rows, H, row_stride);
    else if (D == 64) hipLaunchKernelGGL(ll_bwd_delta_kernel<64>, dim3(grid), dim3(256), 0, s, out, dout, delta, rows, H, row_stride);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_bwd_finish(const BwdFinishParams& p, hipStream_t s) {
    if (p.n_frames <= 0) return hipSuccess;
    const dim3 grid(unsigned(p.n_frames) * unsigned((p.P + 31) / 32), p.H);
    if (p.D == 128) hipLaunchKernelGGL(ll_bwd_finish_kernel<128>, grid, dim3(256), 0, s, p);
    else if (p.D == 64) hipLaunchKernelGGL(ll_bwd_finish_kernel<64>, grid, dim3(256), 0, s, p);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace ll

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

// Direct-to-LDS loads of the streamed fragments through a buffer descriptor: the region's base and the fragment's
// offset stay in scalar registers and a lane contributes only its 16 * lane (the flat form keeps a 64-bit address per
// region in vector registers, which these kernels do not have to spare).  A region of one head is far below 4 GB; the
// descriptor's range covers everything (offsets are in bounds by construction, as with the flat form).
__device__ __forceinline__ __amdgpu_buffer_rsrc_t bw_region(const char* base) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(base), 0, 0x7FFFFFFF, 0x00020000);   // raw buffer of dwords
}
__device__ __forceinline__ void bw_load_lds16(__amdgpu_buffer_rsrc_t r, char* to, int lane_off, int uniform_off) {
    __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (__attribute__((address_space(3))) void*)(to), 16, lane_off, uniform_off, 0, 0);
}

// LDS reads the compiler does not see (it would place each right before its use): the read leaves `dst` pending until
// bw_lds_wait<N>(dst) has run with N = LDS reads issued after it by then (the LDS returns data in issue order; further
// outstanding operations only make the wait longer).  A kernel that uses them must not spill (a spill would store a
// pending register): tests/test_fp8_mfma_operands.py checks the generated code.
__device__ __forceinline__ void bw_lds_read(u32x4& dst, unsigned addr, int offset) {
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(offset));
}
template <int N>
__device__ __forceinline__ void bw_lds_wait(u32x4& x) {
    asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(x) : "n"(N));
}
__device__ __forceinline__ void bw_lds_wait_n(u32x4& x, int n) {
    switch (n) {
        case 0: bw_lds_wait<0>(x); break;
        case 1: bw_lds_wait<1>(x); break;
        case 2: bw_lds_wait<2>(x); break;
        case 3: bw_lds_wait<3>(x); break;
        case 4: bw_lds_wait<4>(x); break;
        case 5: bw_lds_wait<5>(x); break;
        default: bw_lds_wait<0>(x); break;
    }
}

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

// The streamed blocks go from memory straight into a ring of LDS stages (direct-to-LDS loads, one 1 KB fragment per
// wave and load), several blocks ahead of the block being worked on; a stage is overwritten only behind a barrier that
// every wave reaches after its last read of it.
//   dK/dV kernel (a stage is 4 kblock regions + the rows' lse and delta, 32 KB at head_dim 128; 4 stages): per block,
//   wait until this wave's loads of block it have landed, barrier, issue the loads of block it + 3 over the stage of
//   block it - 1, compute.
//   dQ kernel (3 regions, 24 KB; 6 stages): a block reads its own stage and, for the scores of the block after it,
//   the next one.  One barrier per two blocks: wait for everything issued so far (blocks up to it + 2), barrier, issue
//   blocks it + 3 and it + 4 (over the stages of blocks it - 3 and it - 2), compute blocks it and it + 1.
constexpr int BW_DQ_NS = 6;
constexpr int BW_DKV_NS = 4, BW_DKV_PF = BW_DKV_NS - 1;

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
    extern __shared__ __attribute__((aligned(16))) char lds[];   // [BW_DQ_NS][NREG][KB_BYTES]

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
    const __amdgpu_buffer_rsrc_t rsrc[NREG] = {bw_region(src[0]), bw_region(src[1]), bw_region(src[2])};
    auto issue = [&](int kblk, int stage) {
#pragma unroll
        for (int l = 0; l < LPW; ++l) {
            static_assert(FPR == NW && LPW == NREG, "wave w loads fragment w of every region");
            const int region = l, fr = wave_u;
            char* to = lds + (stage * NREG + region) * KB_BYTES + fr * 1024;
            bw_load_lds16(rsrc[region], to, lane * 16, kblk * KB_BYTES + fr * 1024);
        }
    };
    const BwRanges gr = bw_ranges(g);
    BwIter li, ci;
    bw_iter_init(gr, li);
    bw_iter_init(gr, ci);
    constexpr int NS = BW_DQ_NS, PF = 3;              // blocks loaded before the first barrier
#pragma unroll
    for (int j = 0; j < PF; ++j) {
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
    // One block: the vector work and the row-contracting product of block `it` (stage `st`) from its scores (s, dp),
    // and the scores of block it + 1 (stage `st_next`; past the end: the last block again, unused) into (s_next, dp_next).
    // Software pipeline: the score MFMAs of block it + 1 do not depend on the vector work of block it and run under it.
    int st = 0;                                       // it mod NS
    u32x4 fr[4];
    const unsigned lds_lane = (unsigned)(size_t)(__attribute__((address_space(3))) char*)lds + lane * 16;
    auto block = [&](f32x16& s, f32x16& dp, f32x16& s_next, f32x16& dp_next) {
        const int st_next = st + 1 == NS ? 0 : st + 1;

        const int key0 = ci.kb * KBLOCK, cur_rs = ci.rng ? gr.rs1 : gr.rs0, cur_re = ci.rng ? gr.re1 : gr.re0;
        bw_iter_advance(gr, ci);
        if (key0 < cur_rs || key0 + KBLOCK > cur_re)  // uniform: only the blocks at the ends of a range
            bw_kill_dead_rows(s, dp, key0, cur_rs, cur_re, half);

        // The block's 3 KS operand fragments as one sequence, one MFMA each: 2 KS for the scores of block it + 1 (K'
        // and V fragments of stage st_next alternating over ks), then KS for the dQ product of block it (K'^T
        // fragments of stage st).  The reads are issued by hand AHEAD fragments before their MFMA into a ring of RING
        // register buffers (fragment j in buffer j % RING) with counted waits; the compiler's own order put every read
        // right before its MFMA and left the LDS latency exposed.  The vector work of block it (exp2, dZ, packing;
        // independent of the score MFMAs) is dealt out behind them, one register pair per two MFMAs (per MFMA at head_dim 64).
        constexpr int RING = 4, AHEAD = 3, NSC = 2 * KS, NFR = NSC + 2 * DB;
        constexpr int PER = NSC / 8;                  // score MFMAs per (t, e) register pair of the vector work
        static_assert(NSC % 8 == 0, "the vector work's eight register pairs split over the score MFMAs");
        const unsigned next_a = lds_lane + st_next * NREG * KB_BYTES, cur_a = lds_lane + st * NREG * KB_BYTES;
        auto read_frag = [&](int j) {
            if (j < NSC) bw_lds_read(fr[j % RING], next_a, (j & 1) * KB_BYTES + (j >> 1) * 1024);
            else bw_lds_read(fr[j % RING], cur_a, 2 * KB_BYTES + (((j - NSC) % DB) * 2 + (j - NSC) / DB) * 1024);
        };
#pragma unroll
        for (int j = 0; j < AHEAD; ++j) read_frag(j);
#pragma unroll
        for (int r = 0; r < 16; ++r) s_next[r] = dp_next[r] = 0.f;
        unsigned dz[2][4];
#pragma unroll
        for (int j = 0; j < NFR; ++j) {
            if (j + AHEAD < NFR) read_frag(j + AHEAD);
            bw_lds_wait_n(fr[j % RING], NFR - 1 - j < AHEAD ? NFR - 1 - j : AHEAD);
            const bf16x8 a = __builtin_bit_cast(bf16x8, fr[j % RING]);
            if (j < NSC) {
                if (j & 1) dp_next = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, dof[j >> 1], dp_next, 0, 0, 0);
                else s_next = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[j >> 1], s_next, 0, 0, 0);
                if (j % PER == PER - 1) {
                    const int t = (j / PER) / 4, e = (j / PER) % 4;
                    float z[2];
#pragma unroll
                    for (int k = 0; k < 2; ++k) {
                        const int r = 8 * t + 2 * e + k;
                        const float pr = __builtin_amdgcn_exp2f(s[r] - lse);
                        z[k] = pr * (dp[r] - delta);
                    }
                    dz[t][e] = bw_pack_bf16(z[0], z[1]);
                }
            } else {
                const int t = (j - NSC) / DB, db = (j - NSC) % DB;
                const u32x4 bv = {dz[t][0], dz[t][1], dz[t][2], dz[t][3]};
                acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, __builtin_bit_cast(bf16x8, bv), acc[db], 0, 0, 0);
            }
        }
        st = st_next;
    };
    f32x16 s0, dp0, s1, dp1;
    bw_wait_vmcnt<0>();
    bw_barrier();
    scores(lds, s0, dp0);
    for (int it = 0; it < n_blocks; it += 2) {       // two blocks per trip: the two score sets swap roles, no copies
        if (it > 0) {
            bw_wait_vmcnt<0>();
            bw_barrier();
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            int sj = st + 3 + j;
            if (sj >= NS) sj -= NS;
            issue(li.kb, sj);
            bw_iter_advance(gr, li);
        }
        block(s0, dp0, s1, dp1);
        if (it + 1 < n_blocks) block(s1, dp1, s0, dp0);
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
    extern __shared__ __attribute__((aligned(16))) char lds[];   // [BW_DKV_NS][NREG x KB_BYTES | 256]

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
    const __amdgpu_buffer_rsrc_t rsrc[NREG] = {bw_region(src[0]), bw_region(src[1]), bw_region(src[2]), bw_region(src[3])};
    auto issue = [&](int blk_i, int stage) {
#pragma unroll
        for (int l = 0; l < LPW; ++l) {
            static_assert(FPR == NW && LPW == NREG, "wave w loads fragment w of every region");
            const int region = l, fr = wave_u;
            char* to = lds + stage * STAGE_BYTES + region * KB_BYTES + fr * 1024;
            bw_load_lds16(rsrc[region], to, lane * 16, blk_i * KB_BYTES + fr * 1024);
        }
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(aux_src + blk_i * KBLOCK),
                                         (__attribute__((address_space(3))) void*)(lds + stage * STAGE_BYTES + NREG * KB_BYTES), 4, 0, 0);
    };
    constexpr int LOADS = LPW + 1;                    // per wave and block
    constexpr int NS = BW_DKV_NS, PF = BW_DKV_PF;
    static_assert((NS & (NS - 1)) == 0, "stage index by mask");
#pragma unroll
    for (int j = 0; j < PF; ++j) issue(min(qb_begin + j, qb_end - 1), j);

    // One block = 32 operand fragments from LDS, one MFMA each (16 for the two feature-contracting products S and dP,
    // then, behind the vector work that turns them into P and dZ, 16 for the two row-contracting products).  The reads
    // are issued by hand, AHEAD fragments before the MFMA that consumes them, into a ring of RING register buffers,
    // with counted waits (bw_lds_wait<N>: N = reads issued since); the compiler's own order put every read right
    // before its MFMA and left the LDS latency exposed 16 times per block.  Fragment i of a part lives in buffer i % RING;
    // a buffer is read again only behind the MFMA that consumed it.
    constexpr int RING = 4, AHEAD = 3, NF = 2 * KS;   // NF fragments per part
    static_assert(2 * DB * 2 == NF, "both parts have 2 KS fragments");
    u32x4 fr[RING];
    const unsigned lds_lane = (unsigned)(size_t)(__attribute__((address_space(3))) char*)lds + lane * 16;
    // byte offset of fragment i inside a stage: part 0 = q' (K-style), dO (K-style) alternating over ks;
    // part 1 = dO^T, q'^T (V^T-style) alternating over (t, db)
    auto frag_off = [&](int part, int i) constexpr {
        return part == 0 ? (i & 1) * KB_BYTES + (i >> 1) * 1024
                         : (2 + (i & 1)) * KB_BYTES + (((i >> 1) % DB) * 2 + (i >> 1) / DB) * 1024;
    };
    unsigned pw[2][4], dz[2][4];
    f32x16 s, dp;
    // P and dZ of half t of the block's rows from the scores, rounded to bf16 (vector pipe only).  Register r stands
    // for query row0 + 16(r/8) + 8 half + r%8: its lse and delta come from the stage's last 256 bytes, 8 consecutive
    // values per (t, half) (rows past the clip read the zero padding of the two vectors; they are dead rows).
    auto weights = [&](const char* blk, int t) {
        const float* aux = reinterpret_cast<const float*>(blk + NREG * KB_BYTES);
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
    };

    for (int it = 0; it < n_blocks; ++it) {
        bw_wait_vmcnt<(PF - 1) * LOADS>();            // this wave's loads of block it have landed
        bw_barrier();
        issue(min(qb_begin + it + PF, qb_end - 1), (it + PF) & (NS - 1));    // over the stage of block it - 1
        const unsigned st_a = lds_lane + (it & (NS - 1)) * STAGE_BYTES;
        const char* blk = lds + (it & (NS - 1)) * STAGE_BYTES;

        // part 0: S and dP
#pragma unroll
        for (int i = 0; i < AHEAD; ++i) bw_lds_read(fr[i % RING], st_a, frag_off(0, i));
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = dp[r] = 0.f;
#pragma unroll
        for (int i = 0; i < NF; ++i) {
            if (i + AHEAD < NF) bw_lds_read(fr[(i + AHEAD) % RING], st_a, frag_off(0, i + AHEAD));
            bw_lds_wait_n(fr[i % RING], NF - 1 - i < AHEAD ? NF - 1 - i : AHEAD);
            const bf16x8 a = __builtin_bit_cast(bf16x8, fr[i % RING]);
            if (i & 1) dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, vf[i >> 1], dp, 0, 0, 0);
            else s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, kf[i >> 1], s, 0, 0, 0);
        }
        const int row0 = (qb_begin + it) * KBLOCK;
        if (row0 < row_lo || row0 + KBLOCK > row_hi) {   // uniform: only the blocks at the ends of the range
            asm volatile("" ::: "memory");
            bw_kill_dead_rows(s, dp, row0, row_lo, row_hi, half);
        }
        // the first fragments of part 1 are read while the second half of the vector work runs (not earlier: the
        // registers of the scores' first half are free only then)
        weights(blk, 0);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < AHEAD; ++i) bw_lds_read(fr[i % RING], st_a, frag_off(1, i));
        weights(blk, 1);
        __builtin_amdgcn_sched_barrier(0);

        // part 1: dV^T += dO^T P, Gk^T += q'^T dZ; fragment i is (t, db) = ((i / 2) / DB, (i / 2) % DB), dO^T then q'^T
#pragma unroll
        for (int i = 0; i < NF; ++i) {
            if (i + AHEAD < NF) bw_lds_read(fr[(i + AHEAD) % RING], st_a, frag_off(1, i + AHEAD));
            bw_lds_wait_n(fr[i % RING], NF - 1 - i < AHEAD ? NF - 1 - i : AHEAD);
            const bf16x8 a = __builtin_bit_cast(bf16x8, fr[i % RING]);
            const int t = (i >> 1) / DB, db = (i >> 1) % DB;
            if (i & 1) {
                const u32x4 bz = {dz[t][0], dz[t][1], dz[t][2], dz[t][3]};
                acc_k[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, __builtin_bit_cast(bf16x8, bz), acc_k[db], 0, 0, 0);
            } else {
                const u32x4 bp = {pw[t][0], pw[t][1], pw[t][2], pw[t][3]};
                acc_v[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, __builtin_bit_cast(bf16x8, bp), acc_v[db], 0, 0, 0);
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
    const int grid = ((total + 7) / 8) * 8, lds = BW_DQ_NS * 3 * KBLOCK * p.D * 2;
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
    const int grid = ((total + 7) / 8) * 8, lds = BW_DKV_NS * (4 * KBLOCK * p.D * 2 + 256);
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

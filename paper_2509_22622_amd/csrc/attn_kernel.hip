// ll_sink_window_attn / ll_recache_prefill on the GPU: flash-style attention of a
// chunk's rotated queries over the live token-slot ranges of the layer's cache
// (paper Sec. 3.3: sink + short window + current chunk; no mask inside the set).
//
// Formulation per wave: S^T = K Q^T and O^T = V^T P^T with the 32x32x16 bf16 MFMA, so
// that every lane owns ONE query column.  Row max and row sum of the softmax are then
// plain in-lane reductions over accumulator registers; the two lane halves of a query
// are reconciled only when the running reference maximum has to move.  The K and V
// tiles come from HBM already in MFMA-fragment order (see kernels.h), go through LDS
// as straight 16-byte copies and are shared by all waves of the workgroup.
//
// Softmax is computed in fp32 in the log2 domain: p = 2^(s*c - m), c = log2(e)/sqrt(D).
// m is a per-query reference that is raised only when a new score exceeds it by more
// than RESCALE_SLACK (then O and the row sum are rescaled); the final division by the
// row sum makes the result independent of the reference chosen.
#include "kernels.h"

#include <algorithm>
#include <vector>

namespace ll {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

constexpr float RESCALE_SLACK = 6.0f;     // log2 units: p stays below 2^6 between rescales

__device__ inline unsigned pack_bf16(float a, float b) {
    f32x2 v = {a, b};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2));
}

// D: head_dim.  QB: 32-query blocks per wave.  NW: waves per workgroup.  KT: kblocks per tile.
// OCC: waves per SIMD the register allocation must leave room for (several small workgroups per CU).
template <int D, int QB, int NW, int KT, int OCC = 1>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(OCC, 8))) void ll_attn_kernel(const AttnParams p) {
    constexpr int KS = D / 16;                  // MFMA k-steps of the QK^T product
    constexpr int DB = D / 32;                  // 32-row blocks of O^T
    constexpr int KB_BYTES = KBLOCK * D * 2;    // one kblock of K (or of V)
    constexpr int TILE_BYTES = KT * KB_BYTES;
    constexpr int NT = NW * 64;
    constexpr int QT = NW * QB * 32;            // query rows per workgroup
    constexpr int CPT = TILE_BYTES / 16 / NT;   // 16-byte chunks per thread per tile (K, same for V)
    static_assert(TILE_BYTES % (16 * NT) == 0, "tile must split evenly over the threads");

    extern __shared__ __attribute__((aligned(16))) char lds[];   // [2][K tile | V tile]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, half = lane >> 5;

    // Workgroup -> (head, query tile).  Consecutive workgroup ids go round-robin over the
    // 8 XCDs; give each XCD a contiguous run of (head, tile) items so that workgroups that
    // stream the same head's K/V share one L2.
    const int total = p.n_tiles * p.H;
    const int per_xcd = (total + 7) >> 3;
    const int item = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (item >= total) return;
    const int head = item / p.n_tiles;
    const int tile = item % p.n_tiles;
    int ci = 0;
    while (ci + 1 < p.n_chunks && tile >= p.chunk[ci + 1].tile_begin) ++ci;
    const AttnChunk& ch = p.chunk[ci];
    const int q0 = ch.q_begin + (tile - ch.tile_begin) * QT + wave * (QB * 32);

    // Q^T fragments: lane (col, half) holds features 16*ks + 8*half + 0..7 of query q0 + 32n + col.
    bf16x8 qf[QB][KS];
#pragma unroll
    for (int n = 0; n < QB; ++n) {
        const int row = min(q0 + n * 32 + col, ch.q_end - 1);
        const uint16_t* src = p.q + (int64_t(row) * p.H + head) * D + half * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[n][ks] = *reinterpret_cast<const bf16x8*>(src + ks * 16);
    }

    f32x16 o[QB][DB];
    float mref[QB], lsum[QB];
#pragma unroll
    for (int n = 0; n < QB; ++n) {
        mref[n] = -INFINITY;
        lsum[n] = 0.f;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[n][db][r] = 0.f;
    }

    const char* kbase = reinterpret_cast<const char*>(p.k_cache + head * p.head_stride);
    const char* vbase = reinterpret_cast<const char*>(p.v_cache + head * p.head_stride);
    const float c = p.scale_log2e;

    // Tile iterator over the ranges.
    int n_tiles_total = 0;
    for (int r = 0; r < ch.n_ranges; ++r)
        n_tiles_total += ((ch.re[r] + KBLOCK - 1) / KBLOCK - ch.rs[r] / KBLOCK + KT - 1) / KT;
    int rng = 0;
    int kb = ch.rs[0] / KBLOCK;                                   // first kblock of the current tile
    int kb_end = (ch.re[0] + KBLOCK - 1) / KBLOCK;                // end kblock of the current range

    u32x4 kreg[CPT], vreg[CPT];
    auto fetch = [&](int kblk) {
        const char* ks = kbase + int64_t(kblk) * KB_BYTES;
        const char* vs = vbase + int64_t(kblk) * KB_BYTES;
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
            kreg[i] = *reinterpret_cast<const u32x4*>(ks + (tid + i * NT) * 16);
            vreg[i] = *reinterpret_cast<const u32x4*>(vs + (tid + i * NT) * 16);
        }
    };
    auto stash = [&](int buf) {
        char* kd = lds + buf * (2 * TILE_BYTES);
        char* vd = kd + TILE_BYTES;
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
            *reinterpret_cast<u32x4*>(kd + (tid + i * NT) * 16) = kreg[i];
            *reinterpret_cast<u32x4*>(vd + (tid + i * NT) * 16) = vreg[i];
        }
    };

    fetch(kb);
    stash(0);
    __syncthreads();

    for (int it = 0; it < n_tiles_total; ++it) {
        // position of this tile, and of the next one
        const int cur_kb = kb, cur_end = kb_end, cur_rs = ch.rs[rng], cur_re = ch.re[rng];
        kb += KT;
        if (kb >= kb_end && rng + 1 < ch.n_ranges) {
            ++rng;
            kb = ch.rs[rng] / KBLOCK;
            kb_end = (ch.re[rng] + KBLOCK - 1) / KBLOCK;
        }
        const bool more = it + 1 < n_tiles_total;
        if (more) fetch(kb);

        const char* kt = lds + (it & 1) * (2 * TILE_BYTES);
        const char* vt = kt + TILE_BYTES;
#pragma unroll
        for (int kbi = 0; kbi < KT; ++kbi) {
            const int kabs = cur_kb + kbi;
            if (kabs >= cur_end) break;                           // tile reaches past its range
            const int key0 = kabs * KBLOCK;
            const bool edge = key0 < cur_rs || key0 + KBLOCK > cur_re;

            // S^T = K Q^T for 32 keys x (QB*32) queries
            f32x16 s[QB];
#pragma unroll
            for (int n = 0; n < QB; ++n)
#pragma unroll
                for (int r = 0; r < 16; ++r) s[n][r] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const bf16x8 a = *reinterpret_cast<const bf16x8*>(kt + kbi * KB_BYTES + ks * 1024 + lane * 16);
#pragma unroll
                for (int n = 0; n < QB; ++n)
                    s[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[n][ks], s[n], 0, 0, 0);
            }
            // register r of a lane is key key0 + 16*(r/8) + 8*half + r%8
            unsigned live = 0xFFFFu;                              // bit r: key of register r is in range
            if (edge) {
                live = 0;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = key0 + 16 * (r >> 3) + 8 * half + (r & 7);
                    if (key >= cur_rs && key < cur_re) live |= 1u << r;
                }
#pragma unroll
                for (int n = 0; n < QB; ++n)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (!((live >> r) & 1)) s[n][r] = -INFINITY;
            }

            unsigned pb[QB][2][4];                                // P^T fragments, bf16 pairs
#pragma unroll
            for (int n = 0; n < QB; ++n) {
                float mx = s[n][0];
#pragma unroll
                for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[n][r]);
                mx *= c;
                if (__any(mx > mref[n] + RESCALE_SLACK)) {
                    const float both = fmaxf(mx, __shfl_xor(mx, 32));
                    const float mnew = fmaxf(mref[n], both);
                    const float alpha = (mref[n] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mref[n] - mnew);
                    mref[n] = mnew;
                    lsum[n] *= alpha;
#pragma unroll
                    for (int db = 0; db < DB; ++db)
#pragma unroll
                        for (int r = 0; r < 16; ++r) o[n][db][r] *= alpha;
                }
                float pr[16];
                float acc = 0.f;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    pr[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[n][r], c, -mref[n]));
                    acc += pr[r];
                }
                lsum[n] += acc;
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int e = 0; e < 4; ++e) pb[n][t][e] = pack_bf16(pr[8 * t + 2 * e], pr[8 * t + 2 * e + 1]);
            }

            // O^T += V^T P^T
#pragma unroll
            for (int t = 0; t < 2; ++t) {
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    u32x4 av = *reinterpret_cast<const u32x4*>(vt + kbi * KB_BYTES + (db * 2 + t) * 1024 + lane * 16);
                    if (edge) {                                   // dead slots may hold anything, even NaN
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const unsigned b0 = (live >> (8 * t + 2 * e)) & 1, b1 = (live >> (8 * t + 2 * e + 1)) & 1;
                            av[e] &= (b0 ? 0x0000FFFFu : 0u) | (b1 ? 0xFFFF0000u : 0u);
                        }
                    }
                    const bf16x8 a = __builtin_bit_cast(bf16x8, av);
#pragma unroll
                    for (int n = 0; n < QB; ++n) {
                        u32x4 bv = {pb[n][t][0], pb[n][t][1], pb[n][t][2], pb[n][t][3]};
                        o[n][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, __builtin_bit_cast(bf16x8, bv), o[n][db], 0, 0, 0);
                    }
                }
            }
        }

        if (more) stash((it + 1) & 1);
        __syncthreads();
    }

    // out[row][head][32*db + 8*g + 4*half + i] = O^T register 4*g + i, divided by the row sum
#pragma unroll
    for (int n = 0; n < QB; ++n) {
        const float l = lsum[n] + __shfl_xor(lsum[n], 32);
        const float inv = 1.0f / l;
        const int row = q0 + n * 32 + col;
        if (row < ch.q_end) {
            if (p.out_frag != nullptr) {         // uniform: the output projection's operand (kernels.h)
                // features 32 db + 4 G + e and 32 db + 16 + 4 G + e of lane group G are registers 4 g + e of this
                // lane half for g = 0, 2 (G = half) and g = 1, 3 (G = half + 2)
                const int n_ksteps = p.H * DB;
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int hi = 0; hi < 2; ++hi) {
                        const int g0 = hi, g1 = hi + 2;
                        const u32x4 w = {pack_bf16(o[n][db][4 * g0] * inv, o[n][db][4 * g0 + 1] * inv),
                                         pack_bf16(o[n][db][4 * g0 + 2] * inv, o[n][db][4 * g0 + 3] * inv),
                                         pack_bf16(o[n][db][4 * g1] * inv, o[n][db][4 * g1 + 1] * inv),
                                         pack_bf16(o[n][db][4 * g1 + 2] * inv, o[n][db][4 * g1 + 3] * inv)};
                        *reinterpret_cast<u32x4*>(p.out_frag + op_frag_offset(row, head * DB + db, half + 2 * hi, n_ksteps)) = w;
                    }
                continue;
            }
            uint16_t* dst = p.out + (int64_t(row) * p.H + head) * D + half * 4;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    u32x2 w = {pack_bf16(o[n][db][4 * g] * inv, o[n][db][4 * g + 1] * inv),
                               pack_bf16(o[n][db][4 * g + 2] * inv, o[n][db][4 * g + 3] * inv)};
                    *reinterpret_cast<u32x2*>(dst + db * 32 + g * 8) = w;
                }
        }
    }
}

#define LL_VARIANT(D, QB, NW, KT)                                                              \
    { "d" #D "_q" #QB "x" #NW "_k" #KT, D, NW * QB * 32, 2 * 2 * KT * KBLOCK * D * 2,          \
      ll_attn_kernel<D, QB, NW, KT>, NW * 64, KBLOCK }

static const AttnVariant kSimpleVariants[] = {
    LL_VARIANT(128, 2, 4, 2),   // 1: 256 queries, 64-key tiles
    LL_VARIANT(128, 2, 4, 4),   // 2: 256 queries, 128-key tiles
    LL_VARIANT(128, 1, 4, 2),   // 3: 128 queries
    LL_VARIANT(128, 1, 8, 2),   // 4: 256 queries, 8 waves
    LL_VARIANT(64, 2, 4, 2),    // 5
    LL_VARIANT(64, 1, 4, 2),    // 6
    // 128 queries per workgroup and room for 2 or 3 workgroups per CU: for short key sets (cross-attention over a
    // prompt), where a workgroup's life is mostly the load of its queries and the store of its outputs
    { "d128_q1x4_k2_occ2", 128, 128, 2 * 2 * 2 * KBLOCK * 128 * 2, ll_attn_kernel<128, 1, 4, 2, 2>, 256, KBLOCK },   // 7
    { "d128_q1x4_k1_occ3", 128, 128, 2 * 2 * 1 * KBLOCK * 128 * 2, ll_attn_kernel<128, 1, 4, 1, 3>, 256, KBLOCK },   // 8
    { "d64_q1x4_k2_occ2", 64, 128, 2 * 2 * 2 * KBLOCK * 64 * 2, ll_attn_kernel<64, 1, 4, 2, 2>, 256, KBLOCK },       // 9
    { "d64_q1x4_k1_occ3", 64, 128, 2 * 2 * 1 * KBLOCK * 64 * 2, ll_attn_kernel<64, 1, 4, 1, 3>, 256, KBLOCK },       // 10
};
constexpr int kNumSimple = sizeof(kSimpleVariants) / sizeof(kSimpleVariants[0]);
static_assert(kNumSimple == 10, "attn_variant_short_keys names table positions 8 and 10");

// variant ids: 1..kNumSimple are the kernels of this file, then the software-pipelined kernels, then the
// kernels of the 8-bit cache, then the software-pipelined kernels on 16x16x32 MFMAs
static const AttnVariant* variant(int v) {
    if (v >= 1 && v <= kNumSimple) return &kSimpleVariants[v - 1];
    v -= kNumSimple;
    if (v >= 1 && v <= kNumStreamVariants) return &kStreamVariants[v - 1];
    v -= kNumStreamVariants;
    if (v >= 1 && v <= kNumFp8Variants) return &kFp8Variants[v - 1];
    v -= kNumFp8Variants;
    if (v >= 1 && v <= kNumStream16Variants) return &kStream16Variants[v - 1];
    return nullptr;
}
static int first_stream16() { return kNumSimple + kNumStreamVariants + kNumFp8Variants + 1; }
static bool is_stream16(int v) { return v >= first_stream16() && v < first_stream16() + kNumStream16Variants; }
int attn_variant_count() { return kNumSimple + kNumStreamVariants + kNumFp8Variants + kNumStream16Variants; }
const char* attn_variant_name(int v) { return variant(v) ? variant(v)->name : nullptr; }
// the software-pipelined kernels are the default: for the bf16 cache the form built on 16x16x32 MFMAs (faster than the
// 32x32x16 form at every shape measured: 3 to 5 % at head_dim 128, 1 % at 64)
int attn_variant_default(int D, int kblock) {
    if (kblock == KBLOCK8) return kNumSimple + kNumStreamVariants + (D == 128 ? 1 : 2);
    return first_stream16() + (D == 128 ? 0 : 1);
}
int attn_variant_qtile(int v) { return variant(v)->qtile; }
bool attn_variant_supports(int v, int D, int kblock) { return variant(v) && variant(v)->D == D && variant(v)->kblock == kblock; }
// only the software-pipelined bf16 kernels take queries turned back for the sink range (AttnChunk::sink_shift)
bool attn_variant_sink_shift(int v) {
    return (v > kNumSimple && v <= kNumSimple + 2) || (is_stream16(v) && (v < first_stream16() + 2 || (v >= first_stream16() + 6 && v < first_stream16() + 8)));
}
// the software-pipelined kernel that multiplies the queries by AttnParams::scale_log2e itself
int attn_variant_qscale(int D) { return first_stream16() + (D == 128 ? 2 : 3); }
int attn_variant_lse(int D) { return first_stream16() + (D == 128 ? 4 : 5); }
int attn_variant_qrope(int D) { return first_stream16() + (D == 128 ? 8 : 9); }
// the 128-query kernel that leaves room for three workgroups per CU (short key sets, many query tiles)
int attn_variant_short_keys(int D) { return D == 128 ? 8 : 10; }
bool attn_variant_out_frag(int v) { return (v >= 1 && v <= kNumSimple) || is_stream16(v); }
bool attn_variant_applies_scale(int v) {
    return (v >= 1 && v <= kNumSimple) || v == kNumSimple + 3 || v == kNumSimple + 4 || v == first_stream16() + 2 || v == first_stream16() + 3;
}

hipError_t launch_attn(const AttnParams& p_in, int variant, hipStream_t s) {
    if (!attn_variant_supports(variant, p_in.D, p_in.kblock)) return hipErrorInvalidValue;
    AttnParams p = p_in;
    const int KB = p.kblock;
    const AttnVariant& v = *ll::variant(variant);
    const int total = p.n_tiles * p.H;
    if (total <= 0) return hipSuccess;
    for (int c = 0; c < p.n_chunks; ++c) {
        AttnChunk& ch = p.chunk[c];
        ch.n_kblocks = 0;
        for (int r = 0; r < ch.n_ranges; ++r) ch.n_kblocks += (ch.re[r] + KB - 1) / KB - ch.rs[r] / KB;
        if (ch.n_kblocks < 1) return hipErrorInvalidValue;
    }
    int grid = ((total + 7) / 8) * 8;           // the kernels spread their workgroups over the 8 XCDs
    p.n_groups = 0;
    const int groups = p.H * p.n_chunks;
    if (variant > kNumSimple && p.n_chunks > 1 && groups >= 16 && groups <= MAX_XCD_GROUPS) {   // every kernel but the simple ones reads the placement
        // Tiles of different chunks differ in length, and the hardware binds workgroup b to XCD b % 8: hand each
        // XCD whole (head, chunk) groups so that all carry the same number of kblock steps (longest group to the
        // least loaded XCD), and let each start with its longest tiles.
        struct Group { int id, tiles, len; };
        std::vector<Group> all;
        for (int h = 0; h < p.H; ++h)
            for (int c = 0; c < p.n_chunks; ++c) {
                const int tiles = (c + 1 < p.n_chunks ? p.chunk[c + 1].tile_begin : p.n_tiles) - p.chunk[c].tile_begin;
                all.push_back({h * p.n_chunks + c, tiles, p.chunk[c].n_kblocks});
            }
        std::stable_sort(all.begin(), all.end(), [](const Group& a, const Group& b) {
            return int64_t(a.tiles) * a.len > int64_t(b.tiles) * b.len;
        });
        std::vector<Group> per_xcd[8];
        int64_t load[8] = {};
        for (const Group& g : all) {
            const int x = int(std::min_element(load, load + 8) - load);
            per_xcd[x].push_back(g);
            load[x] += int64_t(g.tiles) * g.len;
        }
        int n = 0, most_tiles = 0;
        for (int x = 0; x < 8; ++x) {
            std::stable_sort(per_xcd[x].begin(), per_xcd[x].end(), [](const Group& a, const Group& b) { return a.len > b.len; });
            p.xcd_first[x] = uint16_t(n);
            int tiles = 0;
            for (const Group& g : per_xcd[x]) {
                p.xcd_group[n++] = uint16_t(g.id);
                tiles += g.tiles;
            }
            most_tiles = std::max(most_tiles, tiles);
        }
        p.xcd_first[8] = uint16_t(n);
        p.n_groups = n;
        grid = 8 * most_tiles;
    }
    static bool attr_set[64] = {};
    if (variant > 64) return hipErrorInvalidValue;
    if (!attr_set[variant - 1]) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(v.kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, v.lds_bytes);
        if (e != hipSuccess) return e;
        attr_set[variant - 1] = true;
    }
    hipLaunchKernelGGL(v.kernel, dim3(grid), dim3(v.threads), v.lds_bytes, s, p);
    return hipGetLastError();
}

}  // namespace ll

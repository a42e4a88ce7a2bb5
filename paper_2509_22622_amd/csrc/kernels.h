// Interface between the C-ABI host code and the gfx950 kernels, and the HBM layout
// of the rolling KV cache.
//
// Layout (per layer, per head; all bf16).  Token slots are grouped into "kblocks" of
// 32 slots.  Each kblock is stored as the exact register image the 32x32x16 bf16 MFMA
// wants, so a tile moves HBM -> LDS -> VGPR as straight 16-byte copies:
//   K kblock  [D/8 chunks][32 rows][8 elems]   row i holds key slot 32*b + swap23(i),
//             (swap23 exchanges bits 2 and 3) so that the S^T = K Q^T accumulator
//             registers of a lane hold 8 consecutive keys per half -- the order the
//             P^T operand of the second MFMA needs, with no cross-lane movement.
//   V kblock  [D/32 d-blocks][2 key halves t][2 lane halves h][32 d][8 keys]
//             = V^T fragments: element e of lane (h, dd) is key 32*b + 16*t + 8*h + e
//             at feature 32*db + dd.
// A head's K region is `kblocks_alloc` kblocks long, followed by its V region.
#pragma once
#include <hip/hip_runtime.h>
#include <cmath>
#include <cstdint>

namespace ll {

constexpr int KBLOCK = 32;          // key slots per kblock
constexpr int PAD_KBLOCKS = 8;      // readable padding after the last kblock of a head
constexpr int MAX_RANGES = 3;
constexpr int MAX_ATTN_CHUNKS = 16; // query chunks per attention launch
constexpr int MAX_APPEND_FRAMES = 8;  // frames per cache-write launch (its argument block carries a rotary table per frame)
constexpr int MAX_CHUNK_FRAMES = 32;  // largest chunk (ll_chunk_append splits longer runs of frames into several launches)
constexpr int MAX_T_PAIRS = 24;       // frame-axis rotary pairs: 22 at head_dim 128, 12 at 64
constexpr int MAX_XCD_GROUPS = 256; // (head, chunk) groups an attention launch can place on the XCDs one by one
__host__ __device__ inline int swap23(int i) {
    return (i & ~12) | ((i & 4) << 1) | ((i & 8) >> 1);
}
// Element offset (in bf16 units) of (slot-in-kblock k, feature d) inside a K kblock.
__host__ __device__ inline int k_elem_offset(int k, int d) {
    return (((d >> 3) * 32 + swap23(k)) << 3) + (d & 7);
}
// Element offset of (slot-in-kblock k, feature d) inside a V kblock.
__host__ __device__ inline int v_elem_offset(int k, int d) {
    const int t = k >> 4, h = (k >> 3) & 1, e = k & 7;
    return ((((((d >> 5) * 2 + t) * 2 + h) * 32) + (d & 31)) << 3) + e;
}

// ---- 8-bit (E4M3) cache.  One byte per element, kblocks of 64 slots, stored as the register image of the
// 32x32x64 fp8 MFMA (lane = 32 * k-half + row holds 32 consecutive contraction elements of its k-half), in
// 1 KB pieces [64 lanes][16 bytes] so that HBM -> LDS -> VGPR are straight 16-byte copies:
//   K kblock  [2 row blocks R][D/64 feature halves dh][2 pieces c][lane (h, r)][16]
//             lane (h, r) of piece (R, dh, c) holds key 32R + r, features 64dh + 32h + 16c + 0..15.
//   V kblock  [D/32 d-blocks db][2 pieces R][lane (h, dd)][16]
//             byte 4g + j of lane (h, dd) of piece (db, R) holds key 32R + 8g + 4h + j at feature 32db + dd:
//             the keys whose scores the S^T accumulator registers 4g + j of a lane in half h hold, so the
//             softmax weights go from accumulator to the second MFMA's operand without leaving the lane.
constexpr int KBLOCK8 = 64;
__host__ __device__ inline int k8_byte_offset(int k, int d, int D) {
    const int R = k >> 5, r = k & 31, dh = d >> 6, h = (d >> 5) & 1, c = (d >> 4) & 1;
    return ((((R * (D >> 6) + dh) * 2 + c) * 64 + h * 32 + r) << 4) + (d & 15);
}
__host__ __device__ inline int v8_byte_offset(int k, int d) {
    const int R = k >> 5, r = k & 31, h = (r >> 2) & 1;
    return ((((d >> 5) * 2 + R) * 64 + h * 32 + (d & 31)) << 4) + 4 * (r >> 3) + (r & 3);
}

struct RopeTables {            // device pointers into the cache buffer's tail
    const double* inv_freq_t;  // [n_t]      frame-axis frequencies theta^(-2i/d_t)
    const float2* row_cs;      // [grid_h][n_h]  (cos, sin) of y * freq
    const float2* col_cs;      // [grid_w][n_w]  (cos, sin) of x * freq
    int n_t, n_h, n_w;
};

struct AppendParams {
    const uint16_t* q; const uint16_t* k; const uint16_t* v;   // [n_frames*P, H, D]; q null (bf16 cache only): K, V only
    uint16_t* q_out;                                            // same shape; rotated q times q_scale
    float q_scale;                                              // log2(e) / sqrt(D), folded into q_out
    uint16_t* k_cache; uint16_t* v_cache;                       // layer base (head 0)
    int64_t head_stride;                                        // elements between heads
    RopeTables rope;
    int H, D, P, grid_w;
    int n_frames;
    int64_t frame[MAX_APPEND_FRAMES];                           // absolute frame index (host side: input of set_frame_rotation)
    // (cos, sin) of frame * frequency for every frame-axis pair of every frame, computed on the host in double
    // (set_frame_rotation): the kernels run no trigonometry.  identity != 0: no rotary step at all (every pair
    // passes unchanged; q, where given, only takes q_scale) - the tables are not read then.
    float2 t_cs[MAX_APPEND_FRAMES][MAX_T_PAIRS];
    int identity;
    // When set (bf16 cache): t_cs[0 .. n_frames) is also stored there, [n_frames][MAX_T_PAIRS], for the attention
    // kernels that turn the queries themselves (AttnParams::t_table).
    float2* t_table_out;
    int64_t slot[MAX_APPEND_FRAMES];                            // first token slot
    int seg_begin[MAX_APPEND_FRAMES + 1];                       // prefix sum of kblock segments (32 or 64 slots)
    // 8-bit cache (all null / unused for the bf16 cache): byte pointers, head_stride in bytes
    uint8_t* q8_out; uint8_t* k8_cache; uint8_t* v8_cache;
    float k_mul, v_mul;                                         // 2^-k_exp, 2^-v_exp (q_scale carries 2^k_exp)
};

// Fill p.t_cs from p.frame[0 .. n_frames) and the host copy of the frame-axis frequencies (p.rope.n_t of them).
inline void set_frame_rotation(AppendParams& p, const double* inv_freq_t_host) {
    for (int i = 0; i < p.n_frames; ++i)
        for (int j = 0; j < p.rope.n_t && j < MAX_T_PAIRS; ++j) {
            const double a = double(p.frame[i]) * inv_freq_t_host[j];
            p.t_cs[i][j] = make_float2(float(std::cos(a)), float(std::sin(a)));
        }
}

// One rotary pair (re, im) turned by w = (cos, sin) and scaled, in fp32.  The cache-write kernel and the attention
// kernels that turn their queries on load both go through here, with the contraction fixed by hand, so that they
// produce the same bits.
__device__ __forceinline__ void rope_turn_scaled(float re, float im, float2 w, float scale, float& o_re, float& o_im) {
    const float t = im * w.y, u = im * w.x;
    o_re = __builtin_fmaf(re, w.x, -t) * scale;
    o_im = __builtin_fmaf(re, w.y, u) * scale;
}

struct AttnChunk {
    int q_begin, q_end;          // query rows [q_begin, q_end) of the q tensor
    int tile_begin;              // first query tile of this chunk in the launch
    int n_ranges;
    int rs[MAX_RANGES], re[MAX_RANGES];   // key token-slot ranges
    int n_kblocks;               // kblocks the ranges touch        (filled in by launch_attn)
    // Sink at a fixed rotary distance (0 = off): range 0 is exactly the sink, and its scores are taken with the
    // queries turned back by sink_shift frames on the frame axis of the rotary embedding.
    int sink_shift;
    // Queries given before the rotary embedding (AttnParams::t_table set): row r of the chunk is token (r - q_begin)
    // % P of the frame whose frame-axis (cos, sin) are row t_row + (r - q_begin) / P of the table.
    int t_row;
};

struct AttnParams {
    const uint16_t* q; uint16_t* out;     // [rows, H, D]
    // When set, the output goes here instead, in the fragment order of the output projection (op_frag_offset with
    // H * D / 32 k-steps, the heads side by side); honoured by the kernels attn_variant_out_frag names.  Chunk 0 must
    // start at row 0.
    uint16_t* out_frag;
    const uint16_t* k_cache; const uint16_t* v_cache;   // layer base (head 0)
    int64_t head_stride;
    int H, D;
    float scale_log2e;           // factor still to apply to q.k in the log2 domain (1 when q is pre-scaled); only
                                 // the simple kernels and the *_qscale kernels apply it
    int n_chunks, n_tiles;       // n_tiles = query tiles over all chunks
    // Placement on the 8 XCDs (filled in by launch_attn; workgroup b runs on XCD b % 8).  n_groups == 0: the
    // (head, tile) items are split into 8 contiguous runs.  Otherwise (launches of several chunks, whose tiles
    // differ in length) XCD x runs the (head, chunk) groups xcd_group[xcd_first[x] .. xcd_first[x + 1]) in that
    // order, all tiles of a group on one XCD; group = head * n_chunks + chunk.
    int n_groups;
    // 8-bit cache: E4M3 queries and cache (byte pointers, head_stride in bytes), factor 2^v_exp on the output
    const uint8_t* q8; const uint8_t* k8_cache; const uint8_t* v8_cache;
    float out_scale;
    int kblock;                  // key slots per kblock: 32 (bf16 cache) or 64 (8-bit cache)
    const double* inv_freq_t;    // frame-axis rotary frequencies [n_t] (used when a chunk has a sink_shift)
    int n_t;
    float* lse;                  // *_lse kernels: log2 of each row's sum of 2^score, [H][lse_stride] (null otherwise)
    int64_t lse_stride;
    float* out32;                // *_lse kernels: the output once more in fp32, [rows, H, D] (null: not wanted)
    // *_qrope kernels: q holds the queries as the model's projection made them; a wave turns its rows on load
    // (3D rotary embedding, the same arithmetic as the cache-write kernel) and scales them by q_scale.
    const float2* t_table;       // frame-axis (cos, sin), [frames of the call][MAX_T_PAIRS], written by the cache write
    const float2* row_cs; const float2* col_cs;   // as in RopeTables
    int n_h, n_w, P, grid_w;
    float q_scale;
    uint16_t xcd_first[9];
    uint16_t xcd_group[MAX_XCD_GROUPS];
    AttnChunk chunk[MAX_ATTN_CHUNKS];
};

struct ReadFrameParams {
    const uint16_t* k_cache; const uint16_t* v_cache; int64_t head_stride;
    uint16_t* k_out; uint16_t* v_out;     // [P, H, D], either may be null
    int H, D, P; int64_t slot;
    const uint8_t* k8_cache; const uint8_t* v8_cache;   // 8-bit cache: codes go to k8_out / v8_out
    uint8_t* k8_out; uint8_t* v8_out;
};

// ---- backward pass of the train-time rule (attn_bwd.hip)
constexpr int MAX_BWD_GROUPS = 32;
struct BwdGroup {                // column tiles that share one set of streamed rows
    int c_begin, c_end;          // columns: query rows (dQ kernel) or clip-token indices of keys (dK/dV kernel)
    int tile_begin;              // first tile (bwd_tile_cols columns) of the group in the launch
    int n_ranges;
    int rs[2], re[2];            // streamed rows: key token slots (dQ kernel), query rows (dK/dV kernel: one range)
};
struct BwdParams {
    const uint16_t* q; const uint16_t* dout;            // dQ kernel: rotated, scaled queries and dO, [rows, H, D]
    const float* lse; const float* delta;               // [H][row_stride]
    int64_t row_stride;
    // streamed fragment regions (head 0; element strides between heads): two K-style, two V^T-style
    const uint16_t* s_k1; const uint16_t* s_k2; const uint16_t* s_t1; const uint16_t* s_t2;
    int64_t hs_k1, hs_k2, hs_t1, hs_t2;
    // dK/dV kernel: K-style regions holding the columns' own K' and V rows, and the token slot of clip token 0
    const uint16_t* c_k1; const uint16_t* c_k2;
    int64_t hc_k1, hc_k2, col_slot0;
    float* g1;                   // fp32 [rows, H, D]: Gq (dQ kernel) or Gk (dK/dV kernel)
    uint16_t* dv;                // dK/dV kernel: bf16 [rows, H, D]
    int H, D, n_groups, n_tiles;
    BwdGroup group[MAX_BWD_GROUPS];
};
struct BwdFinishParams {
    const float* gq; const float* gk;                   // [n_frames * P, H, D]
    uint16_t* dq; uint16_t* dk;
    RopeTables rope;
    int H, D, P, grid_w, n_frames;
    int64_t frame0;              // absolute index of the first frame
    float q_mul, k_mul;          // 1/sqrt(D), ln 2
};
int bwd_tile_cols(int D);     // columns per workgroup of the two kernels below
hipError_t launch_bwd_dq(const BwdParams& p, hipStream_t s);
hipError_t launch_bwd_dkv(const BwdParams& p, hipStream_t s);
hipError_t launch_bwd_delta(const float* out32, const uint16_t* dout, float* delta, int rows, int H, int D,
                            int64_t row_stride, hipStream_t s);
hipError_t launch_bwd_finish(const BwdFinishParams& p, hipStream_t s);

// One attention kernel instantiation.
struct AttnVariant {
    const char* name;
    int D, qtile, lds_bytes;
    void (*kernel)(const AttnParams);
    int threads;
    int kblock;                  // 32: bf16 cache, 64: 8-bit cache
};
extern const AttnVariant kStreamVariants[];
extern const int kNumStreamVariants;
extern const AttnVariant kFp8Variants[];
extern const int kNumFp8Variants;
extern const AttnVariant kStream16Variants[];   // the software-pipelined kernels on 16x16x32 MFMAs (attn_stream16.hip)
extern const int kNumStream16Variants;

// Attention variants (query rows per workgroup differ).
int attn_variant_count();
const char* attn_variant_name(int v);
int attn_variant_default(int D, int kblock);
int attn_variant_qtile(int v);                 // query rows per workgroup
bool attn_variant_supports(int v, int D, int kblock);
bool attn_variant_sink_shift(int v);          // the variant honours AttnChunk::sink_shift
int attn_variant_lse(int D);                   // the variant that also writes AttnParams::lse
int attn_variant_qscale(int D);                // the variant for queries not yet scaled (honours scale_log2e)
int attn_variant_short_keys(int D);            // small workgroups, three per CU: for short key sets
int attn_variant_qrope(int D);                 // the variant that turns the queries itself (AttnParams::t_table)
bool attn_variant_applies_scale(int v);        // the variant multiplies the scores (or queries) by scale_log2e itself
bool attn_variant_out_frag(int v);             // the variant honours AttnParams::out_frag

// Output projection y = x w^T (out_proj.hip): x [M, K] and w [N, K] in fragment order, y [M, N] bf16 row-major.
// Fragment order: 16 rows x 32 contraction indices form one 1 KB fragment, ready to be an operand of a 16x16x32 MFMA:
// lane 16 g + r holds, for row 16 b + r, the indices 32 ks + 4 g + 0..3 and 32 ks + 16 + 4 g + 0..3 (the pairing the
// attention kernels' accumulators give for free); the fragments of a row block b lie side by side in ks.  The
// offset, in elements, of the 8 values of (row, k-step ks, lane group g) in a tensor of n_ksteps = K / 32 k-steps:
__host__ __device__ inline int64_t op_frag_offset(int row, int ks, int g, int n_ksteps) {
    return ((int64_t(row >> 4) * n_ksteps + ks) * 64 + 16 * g + (row & 15)) * 8;
}
// x_frag holds ceil(M / 16) row blocks (rows past M in the last one may hold anything); N a multiple of 16, K of 64.
struct OutProjParams { const uint16_t* x_frag; const uint16_t* w_frag; uint16_t* y; int M, N, K; };
hipError_t launch_out_proj(const OutProjParams& p, hipStream_t s);
// w [N, K] bf16 row-major ([output feature][input feature]) -> fragment order, same size
hipError_t launch_pack_out_weight(const uint16_t* w, uint16_t* w_frag, int N, int K, hipStream_t s);

hipError_t launch_append(const AppendParams& p, hipStream_t s);
hipError_t launch_append8(const AppendParams& p, hipStream_t s);
hipError_t launch_read_frame8(const ReadFrameParams& p, hipStream_t s);
hipError_t launch_attn(const AttnParams& p, int variant, hipStream_t s);
hipError_t launch_read_frame(const ReadFrameParams& p, hipStream_t s);
// diagnostic (probe_kernels.hip): sink holds workgroups * 512 floats, counters two 64-bit words; `companion` is the
// kind of instruction issued `per_mfma` (1 or 2) times behind every MFMA
enum ProbeCompanion {
    PROBE_NONE = 0, PROBE_ADD = 1, PROBE_EXP = 2, PROBE_CVT_BF16 = 3, PROBE_DOT2_BF16 = 4, PROBE_MAX3 = 5,
    PROBE_LDS_READ = 6, PROBE_SHAPE_16X16X32 = 7,  // 7: no companion, 16x16x32 MFMAs instead of 32x32x16
    // fp8 32x32x64 MFMAs (E4M3 operands): alone, with what the 8-bit attention kernel issues per MFMA (4 exp2, 4 adds,
    // 2 conversions, 2 max3, two 16-byte LDS reads), with its vector part only, with its LDS part only
    PROBE_FP8_NONE = 8, PROBE_FP8_MIX = 9, PROBE_FP8_VALU = 10, PROBE_FP8_LDS = 11
};
hipError_t launch_probe_mfma(float* sink, unsigned long long* counters, int workgroups, int iters, int random_operands,
                             int companion, int per_mfma, hipStream_t s);

}  // namespace ll

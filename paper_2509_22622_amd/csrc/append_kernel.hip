// ll_chunk_append on the GPU: 3D rotary embedding of the new chunk's Q and K, and the
// write of rotated K and of V into the ring slots of the layer's cache, in the
// MFMA-fragment layout described in kernels.h.  Memory bound; one pass over q, k, v.
//
// Work split: one workgroup per (32-slot segment of a frame, head), heads varying fastest over the workgroups so
// that neighbouring workgroups read neighbouring 256-byte pieces of the same token rows.  A segment is the part of
// one frame that falls into one kblock, so each workgroup owns whole rows of exactly one K kblock and one V kblock
// and builds their images in LDS before storing them with 16-byte stores.
//
// The kernel is a handful of memory round trips long (a chunk is about seven segments per compute unit), so what
// counts is that nothing stands between its start and its loads: a thread first issues every load it will need
// (its rows of q, k and v, the row and column rotary pairs of its tokens), only then touches the data.  The frame
// axis's (cos, sin) come ready-made in the argument block (computed on the host in double, one table per frame).
//
// The rotated queries leave pre-multiplied by log2(e)/sqrt(D) (one rounding of the scaled
// value, so no accuracy is lost): the attention kernel then works in the log2 domain with
// no per-score multiply.
//
// The rotary convention (the paper defines none) is the factorised (frame, row,
// column) form: the D/2 adjacent-element pairs are split n_t | n_h | n_w, pair i of
// an axis turns by position * theta^(-2i/d_axis); frame positions are absolute.
#include "kernels.h"

#include <algorithm>

namespace ll {

typedef unsigned short u16x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

__device__ inline float bf16_to_f32(unsigned short b) { return __uint_as_float(unsigned(b) << 16); }
__device__ inline unsigned short f32_to_bf16(float f) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    f32x2 v = {f, 0.f};
    bf16x2 r = __builtin_convertvector(v, bf16x2);      // v_cvt_pk_bf16_f32, round-to-nearest-even
    return __builtin_bit_cast(unsigned, r) & 0xFFFFu;
}

template <int D>
__global__ __launch_bounds__(256) void ll_append_kernel(const AppendParams p) {
    constexpr int CH = D / 8;                 // 16-byte chunks per (token, head) row
    constexpr int VROW = D + 8;               // padded LDS row (elements)
    constexpr int ITEMS = 32 * CH / 256;      // (token, chunk) items per thread
    __shared__ float2 t_cs[MAX_T_PAIRS];
    __shared__ __attribute__((aligned(16))) unsigned short k_img[32 * D];
    __shared__ __attribute__((aligned(16))) unsigned short v_rows[32 * VROW];

    const int tid = threadIdx.x;
    const int head = blockIdx.x % p.H;
    const int gseg = blockIdx.x / p.H;
    // which frame, which segment
    int fi = 0;
    while (fi + 1 < p.n_frames && gseg >= p.seg_begin[fi + 1]) ++fi;
    const int seg = gseg - p.seg_begin[fi];
    const int64_t slot0 = p.slot[fi];
    const int64_t kb = slot0 / KBLOCK + seg;                       // kblock this segment is in
    const int64_t s_begin = max(slot0, kb * KBLOCK);
    const int64_t s_end = min(slot0 + p.P, (kb + 1) * KBLOCK);
    const int k_lo = int(s_begin - kb * KBLOCK);                   // rows [k_lo, k_hi) of the kblock
    const int k_hi = int(s_end - kb * KBLOCK);
    const int ntok = k_hi - k_lo;
    const int tok0 = int(s_begin - slot0);                         // token inside the frame
    const bool has_q = p.q != nullptr;                             // uniform: keys and values only otherwise
    const bool turn = p.identity == 0;                             // uniform
    const int n_t = p.rope.n_t, n_h = p.rope.n_h;
    const int64_t row0 = int64_t(fi) * p.P + tok0;                 // first input row
    // grid position of the segment's first token: one division per workgroup (the compiler keeps it scalar)
    const int y0 = tok0 / p.grid_w, x0 = tok0 - y0 * p.grid_w;

    // ---- every load first
    u16x8 qv[ITEMS], kv[ITEMS], vv[ITEMS];
    float2 cs[ITEMS][4];
    bool live[ITEMS];
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
        const int item = tid + 256 * it;
        const int ti = item / CH, c = item % CH;
        live[it] = ti < ntok;
        qv[it] = kv[it] = vv[it] = u16x8{};
#pragma unroll
        for (int e = 0; e < 4; ++e) cs[it][e] = make_float2(1.f, 0.f);
        if (live[it]) {
            const int64_t src = ((row0 + ti) * p.H + head) * D + c * 8;
            if (has_q) qv[it] = *reinterpret_cast<const u16x8*>(p.q + src);
            kv[it] = *reinterpret_cast<const u16x8*>(p.k + src);
            vv[it] = *reinterpret_cast<const u16x8*>(p.v + src);
            if (turn) {
                int x = x0 + ti, y = y0;
                if (p.grid_w >= 32) {                              // a segment holds at most 32 tokens: one wrap at most
                    if (x >= p.grid_w) { x -= p.grid_w; ++y; }
                } else {
                    y += x / p.grid_w;
                    x %= p.grid_w;
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int pi = c * 4 + e;
                    if (pi >= n_t) {
                        const float2* src_cs = pi < n_t + n_h ? p.rope.row_cs + (y * n_h + (pi - n_t))
                                                              : p.rope.col_cs + (x * p.rope.n_w + (pi - n_t - n_h));
                        cs[it][e] = *src_cs;
                    }
                }
            }
        }
    }
    if (turn && tid < n_t) t_cs[tid] = p.t_cs[fi][tid];
    if (p.t_table_out != nullptr && blockIdx.x == 0)               // uniform
        for (int i = tid; i < p.n_frames * MAX_T_PAIRS; i += 256)
            p.t_table_out[i] = p.t_cs[i / MAX_T_PAIRS][i % MAX_T_PAIRS];
    __syncthreads();

    // ---- rotation, q' out, K rows and V rows into LDS
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
        if (!live[it]) continue;
        const int item = tid + 256 * it;
        const int ti = item / CH, c = item % CH;
        const int64_t src = ((row0 + ti) * p.H + head) * D + c * 8;
        u16x8 qo, ko;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int pi = c * 4 + e;
            float2 w = cs[it][e];
            if (turn && pi < n_t) w = t_cs[pi];
            const float qr = bf16_to_f32(qv[it][2 * e]), qi = bf16_to_f32(qv[it][2 * e + 1]);
            const float kr = bf16_to_f32(kv[it][2 * e]), ki = bf16_to_f32(kv[it][2 * e + 1]);
            float q_re, q_im;
            rope_turn_scaled(qr, qi, w, p.q_scale, q_re, q_im);
            qo[2 * e] = f32_to_bf16(q_re);
            qo[2 * e + 1] = f32_to_bf16(q_im);
            ko[2 * e] = f32_to_bf16(kr * w.x - ki * w.y);
            ko[2 * e + 1] = f32_to_bf16(kr * w.y + ki * w.x);
        }
        if (!turn) ko = kv[it];                                    // unchanged bit for bit, signed zeros included
        if (has_q) *reinterpret_cast<u16x8*>(p.q_out + src) = qo;
        *reinterpret_cast<u16x8*>(k_img + (c * 32 + swap23(k_lo + ti)) * 8) = ko;
        *reinterpret_cast<u16x8*>(v_rows + (k_lo + ti) * VROW + c * 8) = vv[it];
    }
    __syncthreads();

    // ---- the two images out
    unsigned short* kdst = p.k_cache + head * p.head_stride + kb * (KBLOCK * D);
    unsigned short* vdst = p.v_cache + head * p.head_stride + kb * (KBLOCK * D);
    // K image: unit u is (chunk, row); the row holds key swap23(row)
    for (int u = tid; u < 32 * CH; u += 256) {
        const int key = swap23(u & 31);
        if (key >= k_lo && key < k_hi)
            *reinterpret_cast<u16x8*>(kdst + u * 8) = *reinterpret_cast<const u16x8*>(k_img + u * 8);
    }
    // V image: unit (db, t, h, dd) holds keys 16t + 8h + e, e = 0..7, of feature 32db + dd.  A thread builds the
    // units of two neighbouring features from eight 4-byte LDS reads (one per key: both features at once).
    for (int up = tid; up < 16 * CH; up += 256) {
        const int ddp = up & 15, hh = (up >> 4) & 1, t = (up >> 5) & 1, db = up >> 6;
        const int key0 = 16 * t + 8 * hh;
        const int d = 32 * db + 2 * ddp;
        const int u = ((db * 2 + t) * 2 + hh) * 32 + 2 * ddp;     // unit of feature d; feature d + 1 is unit u + 1
        if (key0 >= k_lo && key0 + 8 <= k_hi) {
            unsigned w[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) w[e] = *reinterpret_cast<const unsigned*>(v_rows + (key0 + e) * VROW + d);
            u32x4 lo, hi;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                lo[e] = __builtin_amdgcn_perm(w[2 * e + 1], w[2 * e], 0x05040100u);    // low halves: feature d
                hi[e] = __builtin_amdgcn_perm(w[2 * e + 1], w[2 * e], 0x07060302u);    // high halves: feature d + 1
            }
            *reinterpret_cast<u32x4*>(vdst + u * 8) = lo;
            *reinterpret_cast<u32x4*>(vdst + (u + 1) * 8) = hi;
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (key0 + e >= k_lo && key0 + e < k_hi) {
                    vdst[u * 8 + e] = v_rows[(key0 + e) * VROW + d];
                    vdst[(u + 1) * 8 + e] = v_rows[(key0 + e) * VROW + d + 1];
                }
        }
    }
}

hipError_t launch_append(const AppendParams& p, hipStream_t s) {
    const int nseg = p.seg_begin[p.n_frames];
    if (nseg <= 0) return hipSuccess;
    if (p.n_frames > MAX_APPEND_FRAMES || (p.identity == 0 && p.rope.n_t > MAX_T_PAIRS)) return hipErrorInvalidValue;
    if (int64_t(nseg) * p.H > 0x7FFFFFFF) return hipErrorInvalidValue;
    dim3 grid(unsigned(nseg) * unsigned(p.H)), block(256);
    if (p.D == 128) hipLaunchKernelGGL(ll_append_kernel<128>, grid, block, 0, s, p);
    else if (p.D == 64) hipLaunchKernelGGL(ll_append_kernel<64>, grid, block, 0, s, p);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

// Copy one frame's K (already rotated) and V out of the cache layout into [P, H, D].
__global__ __launch_bounds__(256) void ll_read_frame_kernel(const ReadFrameParams p) {
    if (p.k_out != nullptr && p.v_out == nullptr) {   // keys only: 8 features of a row are 16 contiguous bytes on both sides
        const int64_t units = int64_t(p.P) * p.H * (p.D / 8);
        for (int64_t u = blockIdx.x * 256LL + threadIdx.x; u < units; u += int64_t(gridDim.x) * 256) {
            const int c = int(u % (p.D / 8));
            const int head = int((u / (p.D / 8)) % p.H);
            const int64_t slot = p.slot + u / (int64_t(p.D / 8) * p.H);
            const int64_t base = head * p.head_stride + (slot / KBLOCK) * (KBLOCK * p.D);
            *reinterpret_cast<u16x8*>(p.k_out + u * 8) =
                *reinterpret_cast<const u16x8*>(p.k_cache + base + k_elem_offset(int(slot % KBLOCK), c * 8));
        }
        return;
    }
    const int64_t n = int64_t(p.P) * p.H * p.D;
    for (int64_t i = blockIdx.x * 256LL + threadIdx.x; i < n; i += int64_t(gridDim.x) * 256) {
        const int d = int(i % p.D);
        const int head = int((i / p.D) % p.H);
        const int64_t tok = i / (int64_t(p.D) * p.H);
        const int64_t slot = p.slot + tok;
        const int64_t base = head * p.head_stride + (slot / KBLOCK) * (KBLOCK * p.D);
        const int k = int(slot % KBLOCK);
        if (p.k_out) p.k_out[i] = p.k_cache[base + k_elem_offset(k, d)];
        if (p.v_out) p.v_out[i] = p.v_cache[base + v_elem_offset(k, d)];
    }
}

hipError_t launch_read_frame(const ReadFrameParams& p, hipStream_t s) {
    const int64_t units = int64_t(p.P) * p.H * (p.D / 8);
    const unsigned grid = unsigned(std::min<int64_t>(std::max<int64_t>((units + 255) / 256, 512), 8192));
    hipLaunchKernelGGL(ll_read_frame_kernel, dim3(grid), dim3(256), 0, s, p);
    return hipGetLastError();
}

}  // namespace ll

// ll_chunk_append on the GPU: 3D rotary embedding of the new chunk's Q and K, and the
// write of rotated K and of V into the ring slots of the layer's cache, in the
// MFMA-fragment layout described in kernels.h.  Memory bound; one pass over q, k, v.
//
// Work split: one workgroup per (32-slot segment of a frame, head).  A segment is the
// part of one frame that falls into one kblock, so each workgroup owns whole rows of
// exactly one K kblock and one V kblock and builds their images in LDS before storing
// them with 16-byte stores.
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
    __shared__ float2 t_cs[64];
    __shared__ __attribute__((aligned(16))) unsigned short k_img[32 * D];
    __shared__ __attribute__((aligned(16))) unsigned short v_rows[32 * VROW];

    const int tid = threadIdx.x;
    const int head = blockIdx.y;
    // which frame, which segment
    int fi = 0;
    while (fi + 1 < p.n_frames && (int)blockIdx.x >= p.seg_begin[fi + 1]) ++fi;
    const int seg = blockIdx.x - p.seg_begin[fi];
    const int64_t slot0 = p.slot[fi];
    const int64_t kb = slot0 / KBLOCK + seg;                       // kblock this segment is in
    const int64_t s_begin = max(slot0, kb * KBLOCK);
    const int64_t s_end = min(slot0 + p.P, (kb + 1) * KBLOCK);
    const int k_lo = int(s_begin - kb * KBLOCK);                   // rows [k_lo, k_hi) of the kblock
    const int k_hi = int(s_end - kb * KBLOCK);
    const int ntok = k_hi - k_lo;
    const int tok0 = int(s_begin - slot0);                         // token inside the frame

    if (tid < p.rope.n_t) {
        double sn, cs;
        sincos(double(p.frame[fi]) * p.rope.inv_freq_t[tid], &sn, &cs);
        t_cs[tid] = make_float2(float(cs), float(sn));
    }
    __syncthreads();

    const int64_t row0 = int64_t(fi) * p.P + tok0;                 // first input row
    for (int item = tid; item < ntok * CH; item += 256) {
        const int ti = item / CH, c = item % CH;
        const int tok = tok0 + ti;
        const int y = tok / p.grid_w, x = tok % p.grid_w;
        const int64_t src = ((row0 + ti) * p.H + head) * D + c * 8;
        const bool has_q = p.q != nullptr;                              // uniform: keys and values only otherwise
        u16x8 qv = {};
        if (has_q) qv = *reinterpret_cast<const u16x8*>(p.q + src);
        const u16x8 kv = *reinterpret_cast<const u16x8*>(p.k + src);
        const u16x8 vv = *reinterpret_cast<const u16x8*>(p.v + src);
        u16x8 qo, ko;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int pi = c * 4 + e;
            float2 cs;
            if (pi < p.rope.n_t) cs = t_cs[pi];
            else if (pi < p.rope.n_t + p.rope.n_h) cs = p.rope.row_cs[y * p.rope.n_h + (pi - p.rope.n_t)];
            else cs = p.rope.col_cs[x * p.rope.n_w + (pi - p.rope.n_t - p.rope.n_h)];
            const float qr = bf16_to_f32(qv[2 * e]), qi = bf16_to_f32(qv[2 * e + 1]);
            const float kr = bf16_to_f32(kv[2 * e]), ki = bf16_to_f32(kv[2 * e + 1]);
            qo[2 * e] = f32_to_bf16((qr * cs.x - qi * cs.y) * p.q_scale);
            qo[2 * e + 1] = f32_to_bf16((qr * cs.y + qi * cs.x) * p.q_scale);
            ko[2 * e] = f32_to_bf16(kr * cs.x - ki * cs.y);
            ko[2 * e + 1] = f32_to_bf16(kr * cs.y + ki * cs.x);
        }
        if (has_q) *reinterpret_cast<u16x8*>(p.q_out + src) = qo;
        *reinterpret_cast<u16x8*>(k_img + (c * 32 + swap23(k_lo + ti)) * 8) = ko;
        *reinterpret_cast<u16x8*>(v_rows + (k_lo + ti) * VROW + c * 8) = vv;
    }
    __syncthreads();

    unsigned short* kdst = p.k_cache + head * p.head_stride + kb * (KBLOCK * D);
    unsigned short* vdst = p.v_cache + head * p.head_stride + kb * (KBLOCK * D);
    for (int u = tid; u < 32 * CH; u += 256) {
        // K image: unit u is (chunk, row); the row holds key swap23(row)
        const int key = swap23(u & 31);
        if (key >= k_lo && key < k_hi)
            *reinterpret_cast<u16x8*>(kdst + u * 8) = *reinterpret_cast<const u16x8*>(k_img + u * 8);
        // V image: unit u is (db, t, h, dd) and holds keys 16t + 8h + e, e = 0..7, of feature 32db + dd
        const int dd = u & 31, hh = (u >> 5) & 1, t = (u >> 6) & 1, db = u >> 7;
        const int key0 = 16 * t + 8 * hh;
        const int d = 32 * db + dd;
        if (key0 >= k_lo && key0 + 8 <= k_hi) {
            u16x8 o;
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = v_rows[(key0 + e) * VROW + d];
            *reinterpret_cast<u16x8*>(vdst + u * 8) = o;
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (key0 + e >= k_lo && key0 + e < k_hi) vdst[u * 8 + e] = v_rows[(key0 + e) * VROW + d];
        }
    }
}

hipError_t launch_append(const AppendParams& p, hipStream_t s) {
    const int nseg = p.seg_begin[p.n_frames];
    if (nseg <= 0) return hipSuccess;
    dim3 grid(nseg, p.H), block(256);
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

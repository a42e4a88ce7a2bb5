// ll_chunk_append for the 8-bit (E4M3) cache: the same 3D rotary embedding as append_kernel.hip (see there for
// the convention), then conversion of the rotated keys, the values and the rotated, pre-scaled queries to E4M3
// and the write of K and V into the ring slots in the fragment layout of the 32x32x64 fp8 MFMA (kernels.h).
// Memory bound; one pass over q, k, v.
//
// Quantisation: e4m3(x) = nearest E4M3 value, ties to even, after clamping |x| to 448 (the hardware conversion
// turns anything beyond 464 into NaN, so the clamp comes first).  K8 = e4m3(K' * 2^-k_exp),
// V8 = e4m3(V * 2^-v_exp), Q8 = e4m3(q' * log2(e)/sqrt(D) * 2^k_exp): the product Q8 . K8 needs no rescaling
// and 2^v_exp is applied once to the attention output.
//
// Work split: one workgroup per (64-slot segment of a frame, head); a segment is the part of one frame that
// falls into one kblock.  The workgroup builds the segment's share of one K kblock and one V kblock in LDS and
// stores whole 16-byte units where the segment covers them, single bytes at a frame boundary inside a unit.
#include "kernels.h"

namespace ll {

typedef unsigned short u16x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

__device__ inline float a8_bf16_to_f32(unsigned short b) { return __uint_as_float(unsigned(b) << 16); }
__device__ inline float a8_clamp(float x) { return fminf(fmaxf(x, -448.0f), 448.0f); }
// four floats -> four E4M3 bytes (byte 0 = a)
__device__ inline unsigned a8_pack4(float a, float b, float c, float d) {
    int w = __builtin_amdgcn_cvt_pk_fp8_f32(a8_clamp(a), a8_clamp(b), 0, false);
    w = __builtin_amdgcn_cvt_pk_fp8_f32(a8_clamp(c), a8_clamp(d), w, true);
    return unsigned(w);
}

template <int D>
__global__ __launch_bounds__(256) void ll_append8_kernel(const AppendParams p) {
    constexpr int CH = D / 8;                 // 8-element chunks per (token, head) row
    constexpr int VROW = D + 16;              // padded LDS row of V bytes
    __shared__ float2 t_cs[64];
    __shared__ __attribute__((aligned(16))) unsigned char k_img[KBLOCK8 * D];
    __shared__ __attribute__((aligned(16))) unsigned char v_rows[KBLOCK8 * VROW];

    const int tid = threadIdx.x;
    const int head = blockIdx.y;
    int fi = 0;
    while (fi + 1 < p.n_frames && (int)blockIdx.x >= p.seg_begin[fi + 1]) ++fi;
    const int seg = blockIdx.x - p.seg_begin[fi];
    const int64_t slot0 = p.slot[fi];
    const int64_t kb = slot0 / KBLOCK8 + seg;                      // kblock this segment is in
    const int64_t s_begin = max(slot0, kb * KBLOCK8);
    const int64_t s_end = min(slot0 + p.P, (kb + 1) * KBLOCK8);
    const int k_lo = int(s_begin - kb * KBLOCK8);                  // slots [k_lo, k_hi) of the kblock
    const int k_hi = int(s_end - kb * KBLOCK8);
    const int ntok = k_hi - k_lo;
    const int tok0 = int(s_begin - slot0);                         // token inside the frame

    if (tid < p.rope.n_t) t_cs[tid] = p.t_cs[fi][tid];           // frame-axis (cos, sin), made on the host in double
    __syncthreads();

    const int64_t row0 = int64_t(fi) * p.P + tok0;                 // first input row
    for (int item = tid; item < ntok * CH; item += 256) {
        const int ti = item / CH, c = item % CH;
        const int tok = tok0 + ti;
        const int y = tok / p.grid_w, x = tok % p.grid_w;
        const int64_t src = ((row0 + ti) * p.H + head) * D + c * 8;
        const u16x8 qv = *reinterpret_cast<const u16x8*>(p.q + src);
        const u16x8 kv = *reinterpret_cast<const u16x8*>(p.k + src);
        const u16x8 vv = *reinterpret_cast<const u16x8*>(p.v + src);
        float qo[8], ko[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int pi = c * 4 + e;
            float2 cs;
            if (pi < p.rope.n_t) cs = t_cs[pi];
            else if (pi < p.rope.n_t + p.rope.n_h) cs = p.rope.row_cs[y * p.rope.n_h + (pi - p.rope.n_t)];
            else cs = p.rope.col_cs[x * p.rope.n_w + (pi - p.rope.n_t - p.rope.n_h)];
            const float qr = a8_bf16_to_f32(qv[2 * e]), qi = a8_bf16_to_f32(qv[2 * e + 1]);
            const float kr = a8_bf16_to_f32(kv[2 * e]), ki = a8_bf16_to_f32(kv[2 * e + 1]);
            qo[2 * e] = (qr * cs.x - qi * cs.y) * p.q_scale;
            qo[2 * e + 1] = (qr * cs.y + qi * cs.x) * p.q_scale;
            ko[2 * e] = (kr * cs.x - ki * cs.y) * p.k_mul;
            ko[2 * e + 1] = (kr * cs.y + ki * cs.x) * p.k_mul;
        }
        const u32x2 q8 = {a8_pack4(qo[0], qo[1], qo[2], qo[3]), a8_pack4(qo[4], qo[5], qo[6], qo[7])};
        const u32x2 k8 = {a8_pack4(ko[0], ko[1], ko[2], ko[3]), a8_pack4(ko[4], ko[5], ko[6], ko[7])};
        float vf[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) vf[e] = a8_bf16_to_f32(vv[e]) * p.v_mul;
        const u32x2 v8 = {a8_pack4(vf[0], vf[1], vf[2], vf[3]), a8_pack4(vf[4], vf[5], vf[6], vf[7])};
        *reinterpret_cast<u32x2*>(p.q8_out + src) = q8;
        *reinterpret_cast<u32x2*>(k_img + k8_byte_offset(k_lo + ti, c * 8, D)) = k8;     // 8 features stay together
        *reinterpret_cast<u32x2*>(v_rows + (k_lo + ti) * VROW + c * 8) = v8;
    }
    __syncthreads();

    unsigned char* kdst = p.k8_cache + head * p.head_stride + kb * (KBLOCK8 * D);
    unsigned char* vdst = p.v8_cache + head * p.head_stride + kb * (KBLOCK8 * D);
    constexpr int UNITS = KBLOCK8 * D / 16;
    for (int u = tid; u < UNITS; u += 256) {
        // K image: unit u = (piece, lane); lane = 32h + r holds key 32R + r of piece (R, dh, c)
        const int piece = u >> 6, r = u & 31;
        const int R = piece / (2 * (D / 64));
        const int key = 32 * R + r;
        if (key >= k_lo && key < k_hi)
            *reinterpret_cast<u32x4*>(kdst + u * 16) = *reinterpret_cast<const u32x4*>(k_img + u * 16);
        // V image: unit u = (db, R, h, dd); byte 4g + j holds key 32R + 8g + 4h + j at feature 32db + dd
        const int dd = u & 31, hh = (u >> 5) & 1, Rv = (u >> 6) & 1, db = u >> 7;
        const int d = 32 * db + dd;
        const int first = 32 * Rv + 4 * hh;                     // keys first + 8g + j
        unsigned w[4];
        bool all = true;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            w[g] = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int kk = first + 8 * g + j;
                const bool in = kk >= k_lo && kk < k_hi;
                all = all && in;
                if (in) w[g] |= unsigned(v_rows[kk * VROW + d]) << (8 * j);
            }
        }
        if (all) {
            const u32x4 o = {w[0], w[1], w[2], w[3]};
            *reinterpret_cast<u32x4*>(vdst + u * 16) = o;
        } else {
#pragma unroll
            for (int g = 0; g < 4; ++g)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int kk = first + 8 * g + j;
                    if (kk >= k_lo && kk < k_hi) vdst[u * 16 + 4 * g + j] = (unsigned char)(w[g] >> (8 * j));
                }
        }
    }
}

hipError_t launch_append8(const AppendParams& p, hipStream_t s) {
    const int nseg = p.seg_begin[p.n_frames];
    if (nseg <= 0) return hipSuccess;
    if (p.n_frames > MAX_APPEND_FRAMES || p.rope.n_t > MAX_T_PAIRS) return hipErrorInvalidValue;
    dim3 grid(nseg, p.H), block(256);
    if (p.D == 128) hipLaunchKernelGGL(ll_append8_kernel<128>, grid, block, 0, s, p);
    else if (p.D == 64) hipLaunchKernelGGL(ll_append8_kernel<64>, grid, block, 0, s, p);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

// Copy one frame's K and V codes out of the cache layout into [P, H, D] bytes.
__global__ __launch_bounds__(256) void ll_read_frame8_kernel(const ReadFrameParams p) {
    const int64_t n = int64_t(p.P) * p.H * p.D;
    for (int64_t i = blockIdx.x * 256LL + threadIdx.x; i < n; i += int64_t(gridDim.x) * 256) {
        const int d = int(i % p.D);
        const int head = int((i / p.D) % p.H);
        const int64_t tok = i / (int64_t(p.D) * p.H);
        const int64_t slot = p.slot + tok;
        const int64_t base = head * p.head_stride + (slot / KBLOCK8) * (KBLOCK8 * p.D);
        const int k = int(slot % KBLOCK8);
        if (p.k8_out) p.k8_out[i] = p.k8_cache[base + k8_byte_offset(k, d, p.D)];
        if (p.v8_out) p.v8_out[i] = p.v8_cache[base + v8_byte_offset(k, d)];
    }
}

hipError_t launch_read_frame8(const ReadFrameParams& p, hipStream_t s) {
    hipLaunchKernelGGL(ll_read_frame8_kernel, dim3(512), dim3(256), 0, s, p);
    return hipGetLastError();
}

}  // namespace ll

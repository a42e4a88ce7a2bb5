// C-ABI, train-time rule (include/longlive.h: ll_clip_*): workspace layout, host bookkeeping and launches.
#include "api_common.h"

using namespace ll;
using namespace ll_api;

extern "C" {

// ---- the train-time rule: forward of a supervised clip over sink + detached window + itself, and its backward pass
struct ll_clip {
    int H, D, P, S, W, T, C, grid_h, grid_w;
    char* dev;                          // null for an index-only handle
    int64_t kb_all, kb_clip;            // kblocks per head region (with readable padding): all frames / clip rows
    int64_t hs_all, hs_clip;            // elements between heads of a fragment region pair
    int64_t row_stride;                 // floats between heads of lse and delta
    // byte offsets into the workspace
    size_t o_a, o_b, o_cq, o_cd, o_qrot, o_krot, o_lse, o_delta, o_gq, o_gk, o_o32, o_zero, o_freq, o_row, o_col;
    RopeTables rope;
    std::vector<double> inv_freq_t;     // host copy of the frame-axis frequencies
    // what the last forward left
    bool have_fwd;
    int64_t ctx_start;
    int n_ctx, n_clip, n_frames;        // n_frames: all resident frames (sink + context + clip)
};

namespace {
struct ClipSizes {
    int64_t kb_all, kb_clip, hs_all, hs_clip, row_stride;
    size_t o_a, o_b, o_cq, o_cd, o_qrot, o_krot, o_lse, o_delta, o_gq, o_gk, o_o32, o_zero, o_freq, o_row, o_col, total;
};
bool clip_shapes_ok(int H, int D, int P, int S, int W, int T, int C) {
    return H >= 1 && H <= 4096 && (D == 64 || D == 128) && P >= 1 && S >= 0 && W >= 0 && T >= 1 && C >= 1 &&
           int64_t(S + W + T) * P < (int64_t(1) << 24);
}
ClipSizes clip_sizes(int H, int D, int P, int S, int W, int T, int C, int grid_h, int grid_w) {
    (void)C;
    ClipSizes z{};
    const int64_t n_all = int64_t(S + W + T) * P, n_clip = int64_t(T) * P;
    z.kb_all = (n_all + KBLOCK - 1) / KBLOCK + PAD_KBLOCKS;
    z.kb_clip = (n_clip + KBLOCK - 1) / KBLOCK + PAD_KBLOCKS;
    z.hs_all = 2 * z.kb_all * KBLOCK * D;
    z.hs_clip = 2 * z.kb_clip * KBLOCK * D;
    z.row_stride = z.kb_clip * KBLOCK;
    size_t off = 0;
    auto take = [&](size_t bytes) { const size_t at = off; off = (off + bytes + 255) & ~size_t(255); return at; };
    z.o_a = take(size_t(z.hs_all) * H * 2);
    z.o_b = take(size_t(z.hs_all) * H * 2);
    z.o_cq = take(size_t(z.hs_clip) * H * 2);
    z.o_cd = take(size_t(z.hs_clip) * H * 2);
    z.o_qrot = take(size_t(n_clip) * H * D * 2);
    z.o_krot = take(size_t(n_all) * H * D * 2);
    z.o_lse = take(size_t(z.row_stride) * H * 4);
    z.o_delta = take(size_t(z.row_stride) * H * 4);
    z.o_gq = take(size_t(n_clip) * H * D * 4);
    z.o_gk = take(size_t(n_clip) * H * D * 4);
    z.o_o32 = take(size_t(n_clip) * H * D * 4);
    const int d_hw = 2 * (D / 6), n_t = (D - 2 * d_hw) / 2, n_h = d_hw / 2;
    z.o_zero = take(size_t(D / 2) * sizeof(double));
    z.o_freq = take(size_t(n_t) * sizeof(double));
    z.o_row = take(size_t(grid_h) * n_h * sizeof(float2));
    z.o_col = take(size_t(grid_w) * n_h * sizeof(float2));
    z.total = off;
    return z;
}
}  // namespace

size_t ll_clip_bytes(int heads, int head_dim, int tokens_per_frame, int sink_frames, int window_frames, int clip_frames,
                     int chunk_frames) {
    if (!clip_shapes_ok(heads, head_dim, tokens_per_frame, sink_frames, window_frames, clip_frames, chunk_frames)) return 0;
    // the rotary tables of any grid with this many tokens fit in 2 * P entries
    return clip_sizes(heads, head_dim, tokens_per_frame, sink_frames, window_frames, clip_frames, chunk_frames,
                      tokens_per_frame, tokens_per_frame).total;
}

ll_status ll_clip_create(int heads, int head_dim, int tokens_per_frame, int sink_frames, int window_frames,
                         int clip_frames, int chunk_frames, int grid_h, int grid_w, float rope_theta, void* dev_buffer,
                         size_t dev_bytes, ll_clip** out) {
    if (!out) return fail(LL_ERR_INVALID_ARG, "out is null");
    *out = nullptr;
    if (!clip_shapes_ok(heads, head_dim, tokens_per_frame, sink_frames, window_frames, clip_frames, chunk_frames))
        return fail(head_dim != 64 && head_dim != 128 && head_dim > 0 ? LL_ERR_UNSUPPORTED : LL_ERR_INVALID_ARG,
                    "bad shape: heads %d head_dim %d (64 or 128) tokens_per_frame %d sink %d window %d clip %d chunk %d",
                    heads, head_dim, tokens_per_frame, sink_frames, window_frames, clip_frames, chunk_frames);
    if (grid_h < 1 || grid_w < 1 || int64_t(grid_h) * grid_w != tokens_per_frame)
        return fail(LL_ERR_INVALID_ARG, "grid %dx%d does not give %d tokens per frame", grid_h, grid_w, tokens_per_frame);
    if (!(rope_theta > 1.0f)) return fail(LL_ERR_INVALID_ARG, "rope_theta must exceed 1");
    const bool index_only = dev_buffer == nullptr && dev_bytes == 0;
    const size_t need = ll_clip_bytes(heads, head_dim, tokens_per_frame, sink_frames, window_frames, clip_frames, chunk_frames);
    const ClipSizes z = clip_sizes(heads, head_dim, tokens_per_frame, sink_frames, window_frames, clip_frames, chunk_frames, grid_h, grid_w);
    ll_clip* c = new ll_clip();
    c->H = heads; c->D = head_dim; c->P = tokens_per_frame; c->S = sink_frames; c->W = window_frames;
    c->T = clip_frames; c->C = chunk_frames; c->grid_h = grid_h; c->grid_w = grid_w;
    c->dev = static_cast<char*>(dev_buffer);
    c->kb_all = z.kb_all; c->kb_clip = z.kb_clip; c->hs_all = z.hs_all; c->hs_clip = z.hs_clip; c->row_stride = z.row_stride;
    c->o_a = z.o_a; c->o_b = z.o_b; c->o_cq = z.o_cq; c->o_cd = z.o_cd; c->o_qrot = z.o_qrot; c->o_krot = z.o_krot;
    c->o_lse = z.o_lse; c->o_delta = z.o_delta; c->o_gq = z.o_gq; c->o_gk = z.o_gk; c->o_o32 = z.o_o32;
    c->o_zero = z.o_zero; c->o_freq = z.o_freq; c->o_row = z.o_row; c->o_col = z.o_col;
    const int d_hw = 2 * (head_dim / 6), n_t = (head_dim - 2 * d_hw) / 2, n_h = d_hw / 2;
    c->rope = RopeTables{nullptr, nullptr, nullptr, n_t, n_h, n_h};
    c->inv_freq_t.resize(n_t);
    for (int i = 0; i < n_t; ++i) c->inv_freq_t[i] = std::pow(double(rope_theta), -2.0 * i / (2.0 * n_t));
    c->have_fwd = false;
    if (!index_only) {
        if (!dev_buffer) { delete c; return fail(LL_ERR_INVALID_ARG, "dev_buffer is null"); }
        if (reinterpret_cast<uintptr_t>(dev_buffer) & 255) { delete c; return fail(LL_ERR_INVALID_ARG, "dev_buffer is not 256-byte aligned"); }
        if (dev_bytes < need) { delete c; return fail(LL_ERR_BUFFER_TOO_SMALL, "dev_buffer has %zu bytes, %zu needed", dev_bytes, need); }
        const std::vector<double>& inv_t = c->inv_freq_t;
        std::vector<float2> row(size_t(grid_h) * n_h), col(size_t(grid_w) * n_h);
        for (int y = 0; y < grid_h; ++y)
            for (int i = 0; i < n_h; ++i) {
                const double a = double(y) * std::pow(double(rope_theta), -2.0 * i / (2.0 * n_h));
                row[size_t(y) * n_h + i] = make_float2(float(std::cos(a)), float(std::sin(a)));
            }
        for (int x = 0; x < grid_w; ++x)
            for (int i = 0; i < n_h; ++i) {
                const double a = double(x) * std::pow(double(rope_theta), -2.0 * i / (2.0 * n_h));
                col[size_t(x) * n_h + i] = make_float2(float(std::cos(a)), float(std::sin(a)));
            }
        hipError_t e = hipMemset(c->dev, 0, z.total);
        if (e == hipSuccess && n_t) e = hipMemcpy(c->dev + z.o_freq, inv_t.data(), inv_t.size() * sizeof(double), hipMemcpyHostToDevice);
        if (e == hipSuccess && !row.empty()) e = hipMemcpy(c->dev + z.o_row, row.data(), row.size() * sizeof(float2), hipMemcpyHostToDevice);
        if (e == hipSuccess && !col.empty()) e = hipMemcpy(c->dev + z.o_col, col.data(), col.size() * sizeof(float2), hipMemcpyHostToDevice);
        if (e == hipSuccess) e = hipDeviceSynchronize();
        if (e != hipSuccess) { delete c; return hip_fail(e, "ll_clip_create: table upload"); }
        c->rope.inv_freq_t = reinterpret_cast<const double*>(c->dev + z.o_freq);
        c->rope.row_cs = reinterpret_cast<const float2*>(c->dev + z.o_row);
        c->rope.col_cs = reinterpret_cast<const float2*>(c->dev + z.o_col);
    }
    *out = c;
    return LL_OK;
}

ll_status ll_clip_destroy(ll_clip* clip) {
    delete clip;
    return LL_OK;
}

extern "C++" {
namespace {
uint16_t* clip_u16(const ll_clip* c, size_t off) { return reinterpret_cast<uint16_t*>(c->dev + off); }
float* clip_f32(const ll_clip* c, size_t off) { return reinterpret_cast<float*>(c->dev + off); }

// Position of frame f in the list of resident frames (sink frames outside the clip first, then context and clip).
int64_t clip_frame_pos(const ll_clip* c, int64_t f) {
    if (c->ctx_start >= c->S) return f < c->S ? f : c->S + (f - c->ctx_start);
    return f;                                                    // first clip of a video: the list starts at frame 0
}

// Key token-slot ranges of the clip chunk [f0, f0 + n): sink, then window and chunk (merged when they touch).
std::vector<SlotRange> clip_key_ranges(const ll_clip* c, int64_t f0, int n) {
    std::vector<SlotRange> r;
    const int64_t sink_end = std::min<int64_t>(c->S, f0 + n);     // sink frames that exist by now
    if (sink_end > 0) r.push_back({0, sink_end * c->P});
    const int64_t lo = std::max<int64_t>(std::max<int64_t>(c->S, f0 - c->W), c->ctx_start);
    if (lo < f0 + n) {
        const SlotRange w{clip_frame_pos(c, lo) * c->P, clip_frame_pos(c, f0 + n - 1) * c->P + c->P};
        if (!r.empty() && r.back().end == w.begin) r.back().end = w.end;
        else r.push_back(w);
    }
    return r;
}

// An identity "rotary step" for the cache-write kernel: every pair on the frame axis at frequency zero.
RopeTables clip_identity_rope(const ll_clip* c) {
    return RopeTables{reinterpret_cast<const double*>(c->dev + c->o_zero), nullptr, nullptr, c->D / 2, 0, 0};
}

// Write `rows` rows of (k, v) as one K-style and one V^T-style region from token slot 0 on, unchanged.
hipError_t clip_write_pair(const ll_clip* c, const uint16_t* k, const uint16_t* v, int64_t rows, uint16_t* region,
                           int64_t kblocks, int64_t head_stride, hipStream_t s) {
    AppendParams p{};
    p.k = k; p.v = v;
    p.k_cache = region; p.v_cache = region + kblocks * KBLOCK * c->D;
    p.head_stride = head_stride;
    p.rope = clip_identity_rope(c);
    p.identity = 1;
    p.H = c->H; p.D = c->D; p.P = int(rows); p.grid_w = int(rows);
    p.n_frames = 1;
    p.frame[0] = 0; p.slot[0] = 0;
    p.seg_begin[0] = 0; p.seg_begin[1] = int((rows + KBLOCK - 1) / KBLOCK);
    return launch_append(p, s);
}
}  // namespace
}  // extern "C++"

ll_status ll_clip_forward(ll_clip* clip, int64_t ctx_start, int n_ctx, int n_clip, const void* q, const void* k,
                          const void* v, void* out, void* stream) {
    if (!clip) return fail(LL_ERR_INVALID_ARG, "clip is null");
    ll_clip* c = clip;
    if (n_clip < 1 || n_clip > c->T) return fail(LL_ERR_INVALID_ARG, "n_clip %d outside [1, %d]", n_clip, c->T);
    if (n_ctx < 0 || n_ctx > c->W) return fail(LL_ERR_INVALID_ARG, "n_ctx %d outside [0, %d]", n_ctx, c->W);
    if (ctx_start < 0) return fail(LL_ERR_INVALID_ARG, "negative ctx_start");
    if (ctx_start != 0 && ctx_start < c->S) return fail(LL_ERR_INVALID_ARG, "ctx_start %lld cuts into the sink [0, %d)", (long long)ctx_start, c->S);
    if (ctx_start == 0 && n_ctx != 0 && c->S > 0) return fail(LL_ERR_INVALID_ARG, "a context starting at frame 0 would contain the sink: pass it as part of the clip");
    if (ctx_start + n_ctx + n_clip > (int64_t(1) << 40)) return fail(LL_ERR_INVALID_ARG, "frame index too large");
    const bool any_null = !q || !k || !v || !out;
    if (c->dev && any_null) return fail(LL_ERR_INVALID_ARG, "null tensor");
    if (!c->dev && !(!q && !k && !v && !out)) return fail(LL_ERR_INVALID_ARG, "index-only handle takes null tensors");
    if (!aligned16(q, k, v, out)) return fail(LL_ERR_INVALID_ARG, "tensors must be 16-byte aligned");
    c->have_fwd = false;
    c->ctx_start = ctx_start; c->n_ctx = n_ctx; c->n_clip = n_clip;
    const int n_sink_outside = ctx_start >= c->S ? c->S : 0;
    c->n_frames = n_sink_outside + n_ctx + n_clip;
    if (!c->dev) { c->have_fwd = true; return LL_OK; }

    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t frame_elems = int64_t(c->P) * c->H * c->D;
    const int64_t clip_start = ctx_start + n_ctx;
    const int first_clip = c->n_frames - n_clip;                  // position of the clip's first frame in the list
    // 1. rotary + cache write of every resident frame into region pair A (K' K-style, V V^T-style); the clip's frames
    //    also give the rotated, scaled queries
    for (int base = 0; base < c->n_frames; base += MAX_APPEND_FRAMES) {
        const int m = std::min(MAX_APPEND_FRAMES, c->n_frames - base);
        for (int part = 0; part < 2; ++part) {                    // frames without queries, then the clip's
            const int lo = part == 0 ? base : std::max(base, first_clip);
            const int hi = part == 0 ? std::min(base + m, first_clip) : base + m;
            if (lo >= hi) continue;
            AppendParams p{};
            p.k = static_cast<const uint16_t*>(k) + lo * frame_elems;
            p.v = static_cast<const uint16_t*>(v) + lo * frame_elems;
            if (part == 1) {
                p.q = static_cast<const uint16_t*>(q) + (lo - first_clip) * frame_elems;
                p.q_out = clip_u16(c, c->o_qrot) + (lo - first_clip) * frame_elems;
            }
            p.q_scale = float(1.4426950408889634 / std::sqrt(double(c->D)));
            p.k_cache = clip_u16(c, c->o_a); p.v_cache = p.k_cache + c->kb_all * KBLOCK * c->D;
            p.head_stride = c->hs_all;
            p.rope = c->rope;
            p.H = c->H; p.D = c->D; p.P = c->P; p.grid_w = c->grid_w;
            p.n_frames = hi - lo;
            p.seg_begin[0] = 0;
            for (int i = 0; i < hi - lo; ++i) {
                const int pos = lo + i;
                p.frame[i] = pos < n_sink_outside ? pos : ctx_start + (pos - n_sink_outside);
                p.slot[i] = int64_t(pos) * c->P;
                p.seg_begin[i + 1] = p.seg_begin[i] + int((p.slot[i] % KBLOCK + c->P + KBLOCK - 1) / KBLOCK);
            }
            set_frame_rotation(p, c->inv_freq_t.data());
            hipError_t e = launch_append(p, s);
            if (e != hipSuccess) return hip_fail(e, "clip cache-write kernel launch");
        }
    }
    // 2. region pair B for the backward pass: V K-style and K'^T V^T-style (K' read back row-major first)
    const int64_t n_all = int64_t(c->n_frames) * c->P;
    {
        ReadFrameParams r{};
        r.k_cache = clip_u16(c, c->o_a); r.v_cache = r.k_cache + c->kb_all * KBLOCK * c->D;
        r.head_stride = c->hs_all;
        r.k_out = clip_u16(c, c->o_krot); r.v_out = nullptr;
        r.H = c->H; r.D = c->D; r.P = int(n_all); r.slot = 0;
        hipError_t e = launch_read_frame(r, s);
        if (e == hipSuccess)
            e = clip_write_pair(c, static_cast<const uint16_t*>(v), clip_u16(c, c->o_krot), n_all, clip_u16(c, c->o_b), c->kb_all, c->hs_all, s);
        if (e != hipSuccess) return hip_fail(e, "clip backward-operand kernels launch");
    }
    // 3. attention of the clip's chunks, each over its own key set, with the row sums kept for the backward pass
    const int variant = attn_variant_lse(c->D);
    const int qt = attn_variant_qtile(variant);
    const int n_chunks = (n_clip + c->C - 1) / c->C;
    for (int base = 0; base < n_chunks; base += MAX_ATTN_CHUNKS) {
        AttnParams p{};
        p.q = clip_u16(c, c->o_qrot); p.out = static_cast<uint16_t*>(out);
        p.k_cache = clip_u16(c, c->o_a); p.v_cache = p.k_cache + c->kb_all * KBLOCK * c->D;
        p.head_stride = c->hs_all;
        p.H = c->H; p.D = c->D; p.kblock = KBLOCK;
        p.scale_log2e = 1.0f;
        p.lse = clip_f32(c, c->o_lse); p.lse_stride = c->row_stride;
        p.out32 = clip_f32(c, c->o_o32);
        const int m = std::min(MAX_ATTN_CHUNKS, n_chunks - base);
        int tiles = 0;
        for (int i = 0; i < m; ++i) {
            const int ci = base + m - 1 - i;                      // longest key sets (the latest chunks) first
            const int64_t f0 = clip_start + int64_t(ci) * c->C;
            const int n = int(std::min<int64_t>(c->C, clip_start + n_clip - f0));
            const std::vector<SlotRange> ranges = clip_key_ranges(c, f0, n);
            AttnChunk& ch = p.chunk[i];
            ch.q_begin = ci * c->C * c->P; ch.q_end = ch.q_begin + n * c->P; ch.tile_begin = tiles;
            ch.n_ranges = int(ranges.size());
            for (int r = 0; r < ch.n_ranges; ++r) { ch.rs[r] = int(ranges[r].begin); ch.re[r] = int(ranges[r].end); }
            tiles += (ch.q_end - ch.q_begin + qt - 1) / qt;
        }
        p.n_chunks = m; p.n_tiles = tiles;
        hipError_t e = launch_attn(p, variant, s);
        if (e != hipSuccess) return hip_fail(e, "clip attention kernel launch");
    }
    c->have_fwd = true;
    return LL_OK;
}

ll_status ll_clip_chunk_key_ranges(const ll_clip* clip, int chunk, int64_t* ranges, int cap, int* n) {
    if (!clip) return fail(LL_ERR_INVALID_ARG, "clip is null");
    if (!n) return fail(LL_ERR_INVALID_ARG, "n is null");
    if (!clip->have_fwd) return fail(LL_ERR_STATE, "no forward pass");
    const int n_chunks = (clip->n_clip + clip->C - 1) / clip->C;
    if (chunk < 0 || chunk >= n_chunks) return fail(LL_ERR_INVALID_ARG, "chunk %d out of range [0, %d)", chunk, n_chunks);
    const int64_t clip_start = clip->ctx_start + clip->n_ctx;
    const int64_t f0 = clip_start + int64_t(chunk) * clip->C;
    const int len = int(std::min<int64_t>(clip->C, clip_start + clip->n_clip - f0));
    const std::vector<SlotRange> r = clip_key_ranges(clip, f0, len);
    *n = int(r.size());
    if (int(r.size()) > cap || (!ranges && !r.empty())) return fail(LL_ERR_BUFFER_TOO_SMALL, "%zu ranges, capacity %d", r.size(), cap);
    for (size_t i = 0; i < r.size(); ++i) { ranges[2 * i] = r[i].begin; ranges[2 * i + 1] = r[i].end; }
    return LL_OK;
}

ll_status ll_clip_backward(ll_clip* clip, const void* dout, void* dq, void* dk, void* dv, void* stream) {
    if (!clip) return fail(LL_ERR_INVALID_ARG, "clip is null");
    ll_clip* c = clip;
    if (!c->have_fwd) return fail(LL_ERR_STATE, "no forward pass to differentiate");
    const bool any_null = !dout || !dq || !dk || !dv;
    if (c->dev && any_null) return fail(LL_ERR_INVALID_ARG, "null tensor");
    if (!c->dev && !(!dout && !dq && !dk && !dv)) return fail(LL_ERR_INVALID_ARG, "index-only handle takes null tensors");
    if (!aligned16(dout, dq, dk, dv)) return fail(LL_ERR_INVALID_ARG, "tensors must be 16-byte aligned");
    if (!c->dev) return LL_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int n_clip = c->n_clip;
    const int64_t rows = int64_t(n_clip) * c->P;
    const int64_t clip_start = c->ctx_start + c->n_ctx;
    const int64_t col_slot0 = int64_t(c->n_frames - n_clip) * c->P;
    const uint16_t* qrot = clip_u16(c, c->o_qrot);
    const uint16_t* dO = static_cast<const uint16_t*>(dout);
    // 1. delta_i = dO_i . O_i (O as the forward kept it, not rounded to bf16), and the clip's q' and dO as fragment
    //    regions (each both ways round)
    hipError_t e = launch_bwd_delta(clip_f32(c, c->o_o32), dO, clip_f32(c, c->o_delta), int(rows), c->H, c->D, c->row_stride, s);
    if (e == hipSuccess) e = clip_write_pair(c, qrot, dO, rows, clip_u16(c, c->o_cq), c->kb_clip, c->hs_clip, s);   // q' K-style, dO^T
    if (e == hipSuccess) e = clip_write_pair(c, dO, qrot, rows, clip_u16(c, c->o_cd), c->kb_clip, c->hs_clip, s);   // dO K-style, q'^T
    if (e != hipSuccess) return hip_fail(e, "clip backward preparation kernels launch");
    const int64_t v_off_all = c->kb_all * KBLOCK * c->D, v_off_clip = c->kb_clip * KBLOCK * c->D;
    const int cols = bwd_tile_cols(c->D);
    // 2. Gq: queries as columns, chunk by chunk over each chunk's key ranges
    const int n_chunks = (n_clip + c->C - 1) / c->C;
    for (int base = 0; base < n_chunks; base += MAX_BWD_GROUPS) {
        BwdParams p{};
        p.q = qrot; p.dout = dO;
        p.lse = clip_f32(c, c->o_lse); p.delta = clip_f32(c, c->o_delta); p.row_stride = c->row_stride;
        p.s_k1 = clip_u16(c, c->o_a); p.hs_k1 = c->hs_all;                    // K'   K-style
        p.s_k2 = clip_u16(c, c->o_b); p.hs_k2 = c->hs_all;                    // V    K-style
        p.s_t1 = clip_u16(c, c->o_b) + v_off_all; p.hs_t1 = c->hs_all;        // K'^T V^T-style
        p.g1 = clip_f32(c, c->o_gq);
        p.H = c->H; p.D = c->D;
        const int m = std::min(MAX_BWD_GROUPS, n_chunks - base);
        int tiles = 0;
        for (int i = 0; i < m; ++i) {
            const int ci = base + m - 1 - i;
            const int64_t f0 = clip_start + int64_t(ci) * c->C;
            const int n = int(std::min<int64_t>(c->C, clip_start + n_clip - f0));
            const std::vector<SlotRange> ranges = clip_key_ranges(c, f0, n);
            BwdGroup& g = p.group[i];
            g.c_begin = ci * c->C * c->P; g.c_end = g.c_begin + n * c->P; g.tile_begin = tiles;
            g.n_ranges = int(ranges.size());
            for (int r = 0; r < g.n_ranges; ++r) { g.rs[r] = int(ranges[r].begin); g.re[r] = int(ranges[r].end); }
            tiles += (g.c_end - g.c_begin + cols - 1) / cols;
        }
        p.n_groups = m; p.n_tiles = tiles;
        e = launch_bwd_dq(p, s);
        if (e != hipSuccess) return hip_fail(e, "dQ kernel launch");
    }
    // 3. Gk and dV: the clip's keys as columns over the query rows of the chunks that see them.  A frame is seen by its
    //    own chunk and by the later chunks that start within W frames after it (a sink frame by all later chunks);
    //    neighbouring frames with the same rows form one group of columns.
    std::vector<BwdGroup> groups;
    for (int gc = 0; gc < n_clip; ++gc) {
        const int64_t gframe = clip_start + gc;
        const int c_first = gc / c->C;
        const int c_last = gframe < c->S ? n_chunks - 1 : std::min(n_chunks - 1, (gc + c->W) / c->C);
        const int rs = c_first * c->C * c->P;
        const int re = int(std::min<int64_t>(n_clip, int64_t(c_last + 1) * c->C) * c->P);
        if (!groups.empty() && groups.back().rs[0] == rs && groups.back().re[0] == re) {
            groups.back().c_end += c->P;
            continue;
        }
        BwdGroup g{};
        g.c_begin = gc * c->P; g.c_end = g.c_begin + c->P;
        g.n_ranges = 1; g.rs[0] = rs; g.re[0] = re;
        groups.push_back(g);
    }
    for (size_t base = 0; base < groups.size(); base += MAX_BWD_GROUPS) {
        BwdParams p{};
        p.lse = clip_f32(c, c->o_lse); p.delta = clip_f32(c, c->o_delta); p.row_stride = c->row_stride;
        p.s_k1 = clip_u16(c, c->o_cq); p.hs_k1 = c->hs_clip;                  // q'   K-style
        p.s_k2 = clip_u16(c, c->o_cd); p.hs_k2 = c->hs_clip;                  // dO   K-style
        p.s_t1 = clip_u16(c, c->o_cq) + v_off_clip; p.hs_t1 = c->hs_clip;     // dO^T V^T-style
        p.s_t2 = clip_u16(c, c->o_cd) + v_off_clip; p.hs_t2 = c->hs_clip;     // q'^T V^T-style
        p.c_k1 = clip_u16(c, c->o_a); p.hc_k1 = c->hs_all;                    // K' of the columns
        p.c_k2 = clip_u16(c, c->o_b); p.hc_k2 = c->hs_all;                    // V  of the columns
        p.col_slot0 = col_slot0;
        p.g1 = clip_f32(c, c->o_gk); p.dv = static_cast<uint16_t*>(dv);
        p.H = c->H; p.D = c->D;
        const int m = int(std::min<size_t>(MAX_BWD_GROUPS, groups.size() - base));
        // longest streams first
        std::vector<BwdGroup> part(groups.begin() + base, groups.begin() + base + m);
        std::stable_sort(part.begin(), part.end(), [](const BwdGroup& a, const BwdGroup& b) { return a.re[0] - a.rs[0] > b.re[0] - b.rs[0]; });
        int tiles = 0;
        for (int i = 0; i < m; ++i) {
            p.group[i] = part[i];
            p.group[i].tile_begin = tiles;
            tiles += (part[i].c_end - part[i].c_begin + cols - 1) / cols;
        }
        p.n_groups = m; p.n_tiles = tiles;
        e = launch_bwd_dkv(p, s);
        if (e != hipSuccess) return hip_fail(e, "dK/dV kernel launch");
    }
    // 4. factors and the turn back through the rotary embedding
    BwdFinishParams f{};
    f.gq = clip_f32(c, c->o_gq); f.gk = clip_f32(c, c->o_gk);
    f.dq = static_cast<uint16_t*>(dq); f.dk = static_cast<uint16_t*>(dk);
    f.rope = c->rope;
    f.H = c->H; f.D = c->D; f.P = c->P; f.grid_w = c->grid_w; f.n_frames = n_clip; f.frame0 = clip_start;
    f.q_mul = float(1.0 / std::sqrt(double(c->D))); f.k_mul = float(0.6931471805599453);
    e = launch_bwd_finish(f, s);
    if (e != hipSuccess) return hip_fail(e, "gradient finish kernel launch");
    return LL_OK;
}

}  // extern "C"

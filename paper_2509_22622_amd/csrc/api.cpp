// C-ABI of the library (see include/longlive.h): argument checks, host bookkeeping and
// kernel launches of the rolling cache (ll_cache_*, ll_chunk_append, ll_sink_window_attn, ll_recache_prefill) and
// the error strings.  The prompt side is in api_prompt.cpp, the train-time rule in api_clip.cpp, the kernel-variant
// knob and the diagnostic probe (include/longlive_diag.h) in api_diag.cpp.  No device memory is allocated here; everything lives in the buffer
// the caller handed to ll_cache_create.
#include <cstdarg>
#include <cstdio>
#include <cstring>

#include "api_common.h"

using namespace ll;
using namespace ll_api;

struct ll_cache {
    int fmt;                // 0: bf16 cache, 1: 8-bit (E4M3) cache
    int kb;                 // key slots per kblock: KBLOCK or KBLOCK8
    int k_exp, v_exp;       // 8-bit cache: K8 = e4m3(K' 2^-k_exp), V8 = e4m3(V 2^-v_exp)
    char* q8_stage;         // 8-bit cache: staging area for the E4M3 queries of a re-prefill
    bool sink_relative;     // the sink keeps a fixed rotary distance to the window (ll_cache_set_sink_relative)
    int layers, H, D;
    Geometry g;
    int grid_h, grid_w;
    double theta;
    char* dev;              // null for an index-only handle
    int64_t kblocks;        // kblocks per head region (with padding)
    int64_t head_stride;    // elements between heads (K region + V region); bytes for the 8-bit cache
    int64_t layer_stride;   // elements between layers
    RopeTables rope;
    float2* t_table;        // bf16 cache: per layer, the frame-axis (cos, sin) of the frames of the last cache write,
    int64_t t_stride;       // [S + W + C][MAX_T_PAIRS], for the attention kernels that turn the queries themselves
    std::vector<double> inv_freq_t;   // host copy of the frame-axis frequencies (the device copy is rope.inv_freq_t)
    std::vector<LayerIndex> layer;
    std::vector<int> staged_t_row;    // per layer: row of t_table at which the staged chunk's frames begin
};

static thread_local std::string g_err;

namespace ll_api {
int g_variant = 0;

ll_status fail(ll_status s, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return s;
}
ll_status hip_fail(hipError_t e, const char* what) {
    return fail(LL_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}
}  // namespace ll_api

namespace {
struct Sizes {
    int64_t kblocks, head_stride, layer_stride, cache_elems;
    int n_t, n_h, n_w;
    size_t stage_off, table_off, row_off, col_off, tt_off, total;
};
bool shapes_ok(int layers, int H, int D, int P, int S, int W, int C) {
    return layers >= 1 && H >= 1 && (D == 64 || D == 128) && P >= 1 && S >= 0 && W >= 0 && C >= 1 &&
           int64_t(S + W + C) * P < (int64_t(1) << 30);
}
Sizes sizes(int fmt, int layers, int H, int D, int P, int S, int W, int C, int grid_h, int grid_w) {
    Sizes z{};
    const int kb = fmt ? KBLOCK8 : KBLOCK;
    const int64_t slots = int64_t(S + W + C) * P;
    z.kblocks = (slots + kb - 1) / kb + PAD_KBLOCKS;
    z.head_stride = 2 * z.kblocks * kb * D;
    z.layer_stride = z.head_stride * H;
    z.cache_elems = z.layer_stride * layers;
    const int d_hw = 2 * (D / 6), d_t = D - 2 * d_hw;
    z.n_t = d_t / 2; z.n_h = d_hw / 2; z.n_w = d_hw / 2;
    size_t off = (size_t(z.cache_elems) * (fmt ? 1 : 2) + 255) & ~size_t(255);
    z.stage_off = off;
    if (fmt) off = (off + size_t(slots) * H * D + 255) & ~size_t(255);   // E4M3 queries of one re-prefill
    z.table_off = off; off += size_t(z.n_t) * sizeof(double);
    off = (off + 255) & ~size_t(255);
    z.row_off = off; off += size_t(grid_h) * z.n_h * sizeof(float2);
    off = (off + 255) & ~size_t(255);
    z.col_off = off; off += size_t(grid_w) * z.n_w * sizeof(float2);
    off = (off + 255) & ~size_t(255);
    z.tt_off = off; off += size_t(layers) * (S + W + C) * MAX_T_PAIRS * sizeof(float2);
    z.total = (off + 255) & ~size_t(255);
    return z;
}
// Staging area of ll_recache_prefill_static: the E4M3 queries of one re-prefill of an 8-bit cache.  One copy per GPU
// the library runs on, held until the process ends.  In host code the array's name is only a stand-in: its device
// address comes from hipGetSymbolAddress, once per device (each GPU has its own copy at its own address).
constexpr size_t STATIC_STAGE_BYTES = size_t(36) << 20;
constexpr int MAX_DEVICES = 64;
static __device__ __align__(256) unsigned char scratch[STATIC_STAGE_BYTES];
static void* g_scratch_ptr[MAX_DEVICES] = {};

// Device address of `scratch` on the current device (looked up on the first call per device).
ll_status static_stage(void** ptr) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= MAX_DEVICES) return fail(LL_ERR_UNSUPPORTED, "device %d beyond the %d the library keeps a staging area for", dev, MAX_DEVICES);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return hip_fail(e, "hipGetSymbolAddress(scratch)");
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return LL_OK;
}
// upper bound of the table area when the grid is not known yet (ll_cache_bytes)
size_t table_bound(int D, int P, int layers, int ring_frames) {
    return 4 * 256 + 64 * sizeof(double) + 2 * size_t(P) * (D / 2) * sizeof(float2) +
           size_t(layers) * ring_frames * MAX_T_PAIRS * sizeof(float2);
}
}  // namespace

extern "C" {

static size_t cache_bytes(int fmt, int layers, int heads, int head_dim, int tokens_per_frame, int sink_frames,
                          int window_frames, int chunk_frames) {
    if (!shapes_ok(layers, heads, head_dim, tokens_per_frame, sink_frames, window_frames, chunk_frames)) return 0;
    Sizes z = sizes(fmt, layers, heads, head_dim, tokens_per_frame, sink_frames, window_frames, chunk_frames, 0, 0);
    return z.table_off + table_bound(head_dim, tokens_per_frame, layers, sink_frames + window_frames + chunk_frames);
}

size_t ll_cache_bytes(int layers, int heads, int head_dim, int tokens_per_frame, int sink_frames,
                      int window_frames, int chunk_frames) {
    return cache_bytes(0, layers, heads, head_dim, tokens_per_frame, sink_frames, window_frames, chunk_frames);
}
size_t ll_cache_bytes_fp8(int layers, int heads, int head_dim, int tokens_per_frame, int sink_frames,
                          int window_frames, int chunk_frames) {
    return cache_bytes(1, layers, heads, head_dim, tokens_per_frame, sink_frames, window_frames, chunk_frames);
}

static ll_status cache_create(int fmt, int k_exp, int v_exp, int layers, int heads, int head_dim, int tokens_per_frame,
                              int sink_frames, int window_frames, int chunk_frames, int grid_h, int grid_w,
                              float rope_theta, void* dev_buffer, size_t dev_bytes, ll_cache** out) {
    if (!out) return fail(LL_ERR_INVALID_ARG, "out is null");
    *out = nullptr;
    if (k_exp < -16 || k_exp > 16 || v_exp < -16 || v_exp > 16)
        return fail(LL_ERR_INVALID_ARG, "k_exp %d or v_exp %d outside [-16, 16]", k_exp, v_exp);
    if (!shapes_ok(layers, heads, head_dim, tokens_per_frame, sink_frames, window_frames, chunk_frames))
        return fail(head_dim != 64 && head_dim != 128 && head_dim > 0 ? LL_ERR_UNSUPPORTED : LL_ERR_INVALID_ARG,
                    "bad shape: layers %d heads %d head_dim %d (64 or 128) tokens_per_frame %d sink %d window %d chunk %d",
                    layers, heads, head_dim, tokens_per_frame, sink_frames, window_frames, chunk_frames);
    if (grid_h < 1 || grid_w < 1 || int64_t(grid_h) * grid_w != tokens_per_frame)
        return fail(LL_ERR_INVALID_ARG, "grid %dx%d does not give %d tokens per frame", grid_h, grid_w, tokens_per_frame);
    if (!(rope_theta > 1.0f)) return fail(LL_ERR_INVALID_ARG, "rope_theta must exceed 1");
    if (chunk_frames > MAX_CHUNK_FRAMES)
        return fail(LL_ERR_UNSUPPORTED, "chunk_frames above %d", MAX_CHUNK_FRAMES);
    const bool index_only = dev_buffer == nullptr && dev_bytes == 0;
    const size_t need = cache_bytes(fmt, layers, heads, head_dim, tokens_per_frame, sink_frames, window_frames, chunk_frames);
    if (!index_only) {
        if (!dev_buffer) return fail(LL_ERR_INVALID_ARG, "dev_buffer is null");
        if (reinterpret_cast<uintptr_t>(dev_buffer) & 255) return fail(LL_ERR_INVALID_ARG, "dev_buffer is not 256-byte aligned");
        if (dev_bytes < need) return fail(LL_ERR_BUFFER_TOO_SMALL, "dev_buffer has %zu bytes, %zu needed", dev_bytes, need);
    }
    Sizes z = sizes(fmt, layers, heads, head_dim, tokens_per_frame, sink_frames, window_frames, chunk_frames, grid_h, grid_w);
    ll_cache* c = new ll_cache();
    c->fmt = fmt; c->kb = fmt ? KBLOCK8 : KBLOCK; c->k_exp = k_exp; c->v_exp = v_exp;
    c->sink_relative = false;
    c->q8_stage = (fmt && dev_buffer) ? static_cast<char*>(dev_buffer) + z.stage_off : nullptr;
    c->layers = layers; c->H = heads; c->D = head_dim;
    c->g.P = tokens_per_frame; c->g.S = sink_frames; c->g.W = window_frames; c->g.C = chunk_frames;
    c->grid_h = grid_h; c->grid_w = grid_w; c->theta = rope_theta;
    c->dev = static_cast<char*>(dev_buffer);
    c->kblocks = z.kblocks; c->head_stride = z.head_stride; c->layer_stride = z.layer_stride;
    c->layer.assign(layers, LayerIndex());
    c->staged_t_row.assign(layers, 0);
    c->rope = RopeTables{nullptr, nullptr, nullptr, z.n_t, z.n_h, z.n_w};
    if (z.n_t > MAX_T_PAIRS) { delete c; return fail(LL_ERR_UNSUPPORTED, "%d frame-axis rotary pairs, at most %d", z.n_t, MAX_T_PAIRS); }
    c->inv_freq_t.resize(z.n_t);
    for (int i = 0; i < z.n_t; ++i) c->inv_freq_t[i] = std::pow(double(rope_theta), -2.0 * i / (2.0 * z.n_t));
    if (!index_only) {
        // Rotary tables: angles in double, stored as float (cos, sin); frame frequencies stay double.
        const std::vector<double>& inv_t = c->inv_freq_t;
        std::vector<float2> row(size_t(grid_h) * z.n_h), col(size_t(grid_w) * z.n_w);
        for (int y = 0; y < grid_h; ++y)
            for (int i = 0; i < z.n_h; ++i) {
                const double a = double(y) * std::pow(double(rope_theta), -2.0 * i / (2.0 * z.n_h));
                row[size_t(y) * z.n_h + i] = make_float2(float(std::cos(a)), float(std::sin(a)));
            }
        for (int x = 0; x < grid_w; ++x)
            for (int i = 0; i < z.n_w; ++i) {
                const double a = double(x) * std::pow(double(rope_theta), -2.0 * i / (2.0 * z.n_w));
                col[size_t(x) * z.n_w + i] = make_float2(float(std::cos(a)), float(std::sin(a)));
            }
        hipError_t e = hipMemset(c->dev, 0, need);      // all of it: the padding behind the tables too
        if (e == hipSuccess) e = hipMemcpy(c->dev + z.table_off, inv_t.data(), inv_t.size() * sizeof(double), hipMemcpyHostToDevice);
        if (e == hipSuccess && !row.empty()) e = hipMemcpy(c->dev + z.row_off, row.data(), row.size() * sizeof(float2), hipMemcpyHostToDevice);
        if (e == hipSuccess && !col.empty()) e = hipMemcpy(c->dev + z.col_off, col.data(), col.size() * sizeof(float2), hipMemcpyHostToDevice);
        if (e == hipSuccess) e = hipDeviceSynchronize();
        if (e != hipSuccess) { delete c; return hip_fail(e, "ll_cache_create: table upload"); }
        c->rope.inv_freq_t = reinterpret_cast<const double*>(c->dev + z.table_off);
        c->rope.row_cs = reinterpret_cast<const float2*>(c->dev + z.row_off);
        c->rope.col_cs = reinterpret_cast<const float2*>(c->dev + z.col_off);
        c->t_table = reinterpret_cast<float2*>(c->dev + z.tt_off);
        c->t_stride = int64_t(sink_frames + window_frames + chunk_frames) * MAX_T_PAIRS;
    }
    *out = c;
    return LL_OK;
}

ll_status ll_cache_create(int layers, int heads, int head_dim, int tokens_per_frame, int sink_frames,
                          int window_frames, int chunk_frames, int grid_h, int grid_w, float rope_theta,
                          void* dev_buffer, size_t dev_bytes, ll_cache** out) {
    return cache_create(0, 0, 0, layers, heads, head_dim, tokens_per_frame, sink_frames, window_frames, chunk_frames,
                        grid_h, grid_w, rope_theta, dev_buffer, dev_bytes, out);
}
ll_status ll_cache_create_fp8(int layers, int heads, int head_dim, int tokens_per_frame, int sink_frames,
                              int window_frames, int chunk_frames, int grid_h, int grid_w, float rope_theta,
                              int k_exp, int v_exp, void* dev_buffer, size_t dev_bytes, ll_cache** out) {
    return cache_create(1, k_exp, v_exp, layers, heads, head_dim, tokens_per_frame, sink_frames, window_frames,
                        chunk_frames, grid_h, grid_w, rope_theta, dev_buffer, dev_bytes, out);
}

ll_status ll_cache_destroy(ll_cache* cache) {
    delete cache;
    return LL_OK;
}

#define CHECK_CACHE_LAYER(cache, layer)                                             \
    if (!(cache)) return fail(LL_ERR_INVALID_ARG, "cache is null");                 \
    if ((layer) < 0 || (layer) >= (cache)->layers)                                  \
        return fail(LL_ERR_INVALID_ARG, "layer %d out of range [0, %d)", (layer), (cache)->layers)

ll_status ll_cache_reset(ll_cache* cache, int layer) {
    if (!cache) return fail(LL_ERR_INVALID_ARG, "cache is null");
    if (layer < -1 || layer >= cache->layers) return fail(LL_ERR_INVALID_ARG, "layer %d out of range", layer);
    for (int l = 0; l < cache->layers; ++l)
        if (layer < 0 || l == layer) cache->layer[l] = LayerIndex();
    return LL_OK;
}

static uint16_t* layer_k(const ll_cache* c, int layer) {
    return reinterpret_cast<uint16_t*>(c->dev) + int64_t(layer) * c->layer_stride;
}
static uint16_t* layer_v(const ll_cache* c, int layer) {
    return layer_k(c, layer) + c->kblocks * KBLOCK * c->D;
}
static uint8_t* layer_k8(const ll_cache* c, int layer) {
    return reinterpret_cast<uint8_t*>(c->dev) + int64_t(layer) * c->layer_stride;
}
static uint8_t* layer_v8(const ll_cache* c, int layer) {
    return layer_k8(c, layer) + c->kblocks * KBLOCK8 * c->D;
}

// Enqueue the rotary + cache write of `n` frames whose absolute indices are frames[i];
// rows of q/k/v are consecutive frames.
static ll_status enqueue_append(ll_cache* c, int layer, const int64_t* frames, int n, const void* q, const void* k,
                                const void* v, void* q_out, hipStream_t s) {
    const int64_t frame_elems = int64_t(c->g.P) * c->H * c->D;
    for (int base = 0; base < n; base += MAX_APPEND_FRAMES) {
        AppendParams p{};
        const int m = std::min(MAX_APPEND_FRAMES, n - base);
        p.q = q ? static_cast<const uint16_t*>(q) + base * frame_elems : nullptr;       // null: keys and values only
        p.k = static_cast<const uint16_t*>(k) + base * frame_elems;
        p.v = static_cast<const uint16_t*>(v) + base * frame_elems;
        p.q_scale = float(1.4426950408889634 / std::sqrt(double(c->D)));
        if (c->fmt) {
            p.q8_out = static_cast<uint8_t*>(q_out) + base * frame_elems;
            p.k8_cache = layer_k8(c, layer); p.v8_cache = layer_v8(c, layer);
            p.q_scale = std::ldexp(p.q_scale, c->k_exp);
            p.k_mul = std::ldexp(1.0f, -c->k_exp); p.v_mul = std::ldexp(1.0f, -c->v_exp);
        } else {
            p.q_out = q_out ? static_cast<uint16_t*>(q_out) + base * frame_elems : nullptr;
            p.k_cache = layer_k(c, layer); p.v_cache = layer_v(c, layer);
            if (base + m <= c->t_stride / MAX_T_PAIRS) p.t_table_out = c->t_table + layer * c->t_stride + base * MAX_T_PAIRS;
        }
        p.head_stride = c->head_stride;
        p.rope = c->rope;
        p.H = c->H; p.D = c->D; p.P = c->g.P; p.grid_w = c->grid_w;
        p.n_frames = m;
        p.seg_begin[0] = 0;
        for (int i = 0; i < m; ++i) {
            p.frame[i] = frames[base + i];
            p.slot[i] = slot_of_frame(c->g, frames[base + i]);
            const int nseg = int((p.slot[i] % c->kb + c->g.P + c->kb - 1) / c->kb);
            p.seg_begin[i + 1] = p.seg_begin[i] + nseg;
        }
        set_frame_rotation(p, c->inv_freq_t.data());
        hipError_t e = c->fmt ? launch_append8(p, s) : launch_append(p, s);
        if (e != hipSuccess) return hip_fail(e, "append kernel launch");
    }
    return LL_OK;
}

static int pick_variant(const ll_cache* c) {
    // (the kernel that turns its queries itself is chosen by the calls that hand it unrotated queries, never forced)
    if (g_variant != 0 && attn_variant_supports(g_variant, c->D, c->kb) && g_variant != attn_variant_qrope(c->D)) return g_variant;
    return attn_variant_default(c->D, c->kb);
}

struct ChunkWork { int q_begin, q_end; std::vector<SlotRange> ranges; int64_t f0; int t_row = 0; };

// Frames by which the queries of a chunk starting at f0 are turned back for the sink's scores (0: plain rule).
static int64_t sink_shift_of(const ll_cache* c, int64_t f0) {
    if (!c->sink_relative || c->g.S == 0) return 0;
    return std::max<int64_t>(0, f0 - c->g.W - c->g.S);
}

// Turn a list of query chunks (each with its key ranges) into kernel launches: every check that can fail is made
// here, before anything is enqueued or any bookkeeping changes.
struct AttnLaunches { int variant = 0; std::vector<AttnParams> params; };

// The queries can be turned by the attention kernel itself (then the cache write before it takes keys and values
// only): bf16 cache, the default kernel, no chunk whose sink is scored with turned-back queries.
static bool can_turn_queries(const ll_cache* c, const std::vector<ChunkWork>& work);

// raw_q: q holds the queries before the rotary embedding; chunk i's frames are rows work[i].t_row .. of the table the
// cache write of the same call (or, for a staged chunk, the last ll_chunk_append) left for the layer.
static ll_status build_attn(const ll_cache* c, int layer, const std::vector<ChunkWork>& work, const void* q, void* out,
                            AttnLaunches& L, bool raw_q = false) {
    const int variant = raw_q ? attn_variant_qrope(c->D) : pick_variant(c);
    const int qt = attn_variant_qtile(variant);
    L.variant = variant;
    L.params.clear();
    for (size_t base = 0; base < work.size(); base += MAX_ATTN_CHUNKS) {
        AttnParams p{};
        p.out = static_cast<uint16_t*>(out);
        p.kblock = c->kb;
        if (c->fmt) {
            p.q8 = static_cast<const uint8_t*>(q);
            p.k8_cache = layer_k8(c, layer); p.v8_cache = layer_v8(c, layer);
            p.out_scale = std::ldexp(1.0f, c->v_exp);
        } else {
            p.q = static_cast<const uint16_t*>(q);
            p.k_cache = layer_k(c, layer); p.v_cache = layer_v(c, layer);
        }
        p.head_stride = c->head_stride;
        p.H = c->H; p.D = c->D;
        p.scale_log2e = 1.0f;          // ll_chunk_append already folded log2(e)/sqrt(D) into q
        if (raw_q) {
            p.t_table = c->t_table + layer * c->t_stride;
            p.row_cs = c->rope.row_cs; p.col_cs = c->rope.col_cs;
            p.n_h = c->rope.n_h; p.n_w = c->rope.n_w; p.P = c->g.P; p.grid_w = c->grid_w;
            p.q_scale = float(1.4426950408889634 / std::sqrt(double(c->D)));
        }
        const int m = int(std::min<size_t>(MAX_ATTN_CHUNKS, work.size() - base));
        // longest key sets first: they bound the launch
        std::vector<int> order(m);
        for (int i = 0; i < m; ++i) order[i] = int(base) + i;
        auto keys = [&](int i) { int64_t t = 0; for (auto& r : work[i].ranges) t += r.end - r.begin; return t; };
        std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return keys(a) > keys(b); });
        p.inv_freq_t = c->rope.inv_freq_t; p.n_t = c->rope.n_t;
        int tiles = 0;
        for (int i = 0; i < m; ++i) {
            ChunkWork w = work[order[i]];
            const int64_t shift = sink_shift_of(c, w.f0);
            if (shift != 0) {
                // the sink's scores use other queries than the rest: the sink must be a range of its own
                if (!attn_variant_sink_shift(variant)) return fail(LL_ERR_UNSUPPORTED, "attention variant %d has no sink-relative mode", variant);
                if (shift > 0x7FFFFFFF) return fail(LL_ERR_UNSUPPORTED, "sink shift %lld too large", (long long)shift);
                const int64_t sink_end = int64_t(c->g.S) * c->g.P;
                if (w.ranges.empty() || w.ranges[0].begin != 0 || w.ranges[0].end < sink_end)
                    return fail(LL_ERR_STATE, "sink frames are not the first key range");
                if (w.ranges[0].end > sink_end) {
                    w.ranges.insert(w.ranges.begin() + 1, SlotRange{sink_end, w.ranges[0].end});
                    w.ranges[0].end = sink_end;
                }
            }
            if (w.ranges.empty() || w.ranges.size() > size_t(MAX_RANGES))
                return fail(LL_ERR_STATE, "key set has %zu ranges", w.ranges.size());
            AttnChunk& ch = p.chunk[i];
            ch.q_begin = w.q_begin; ch.q_end = w.q_end; ch.tile_begin = tiles;
            ch.sink_shift = int(shift);
            ch.t_row = w.t_row;
            ch.n_ranges = int(w.ranges.size());
            for (int r = 0; r < ch.n_ranges; ++r) { ch.rs[r] = int(w.ranges[r].begin); ch.re[r] = int(w.ranges[r].end); }
            tiles += (w.q_end - w.q_begin + qt - 1) / qt;
        }
        p.n_chunks = m; p.n_tiles = tiles;
        L.params.push_back(p);
    }
    return LL_OK;
}

static bool can_turn_queries(const ll_cache* c, const std::vector<ChunkWork>& work) {
    if (c->fmt || g_variant != 0) return false;
    for (const ChunkWork& w : work)
        if (sink_shift_of(c, w.f0) != 0) return false;
    return true;
}

static ll_status launch_built_attn(const AttnLaunches& L, hipStream_t s) {
    for (const AttnParams& p : L.params) {
        hipError_t e = launch_attn(p, L.variant, s);
        if (e != hipSuccess) return hip_fail(e, "attention kernel launch");
    }
    return LL_OK;
}

ll_status ll_chunk_append(ll_cache* cache, int layer, int64_t frame_start, int n_frames, const void* q, const void* k,
                          const void* v, void* q_out, void* stream) {
    CHECK_CACHE_LAYER(cache, layer);
    if (n_frames < 1 || n_frames > cache->g.C)
        return fail(LL_ERR_INVALID_ARG, "n_frames %d outside [1, %d]", n_frames, cache->g.C);
    if (frame_start < 0) return fail(LL_ERR_INVALID_ARG, "negative frame_start");
    // q and q_out both null: keys and values only (the queries then go, unrotated, to ll_sink_window_attn_unrotated)
    const bool kv_only = cache->dev && !q && !q_out && k && v;
    if (kv_only && cache->fmt) return fail(LL_ERR_UNSUPPORTED, "the 8-bit cache takes its queries in ll_chunk_append");
    const bool any_null = !q || !k || !v || !q_out;
    if (cache->dev && any_null && !kv_only) return fail(LL_ERR_INVALID_ARG, "null tensor");
    if (!cache->dev && !(!q && !k && !v && !q_out)) return fail(LL_ERR_INVALID_ARG, "index-only handle takes null tensors");
    if (!aligned16(q, k, v, q_out)) return fail(LL_ERR_INVALID_ARG, "tensors must be 16-byte aligned");
    if (cache->fmt && cache->dev && (q_out == q || q_out == k || q_out == v))
        return fail(LL_ERR_INVALID_ARG, "q_out (E4M3 bytes) must not alias q, k or v");
    LayerIndex& L = cache->layer[layer];
    if (classify_append(L, frame_start) == AppendKind::Invalid)
        return fail(LL_ERR_STATE, "layer %d: frame_start %lld neither repeats (%lld) nor follows (%lld) the staged chunk",
                    layer, (long long)frame_start, (long long)L.staged_f0, (long long)(L.staged_f0 + L.staged_n));
    if (cache->dev) {
        int64_t frames[MAX_CHUNK_FRAMES];
        for (int i = 0; i < n_frames; ++i) frames[i] = frame_start + i;
        ll_status st = enqueue_append(cache, layer, frames, n_frames, q, k, v, q_out, static_cast<hipStream_t>(stream));
        if (st != LL_OK) return st;
    }
    apply_append(cache->g, L, frame_start, n_frames);
    cache->staged_t_row[layer] = 0;
    return LL_OK;
}

ll_status ll_sink_window_attn(ll_cache* cache, int layer, const void* q_roped, void* out, void* stream) {
    CHECK_CACHE_LAYER(cache, layer);
    if (!cache->dev) return fail(LL_ERR_INVALID_ARG, "index-only handle has no device cache");
    if (!q_roped || !out) return fail(LL_ERR_INVALID_ARG, "null tensor");
    if (!aligned16(q_roped, out)) return fail(LL_ERR_INVALID_ARG, "tensors must be 16-byte aligned");
    const LayerIndex& L = cache->layer[layer];
    if (L.staged_n == 0) return fail(LL_ERR_STATE, "layer %d: no staged chunk", layer);
    std::vector<ChunkWork> work(1);
    work[0].q_begin = 0;
    work[0].q_end = L.staged_n * cache->g.P;
    work[0].ranges = live_ranges(cache->g, L);
    work[0].f0 = L.staged_f0;
    AttnLaunches launches;
    ll_status st = build_attn(cache, layer, work, q_roped, out, launches);
    if (st != LL_OK) return st;
    return launch_built_attn(launches, static_cast<hipStream_t>(stream));
}

ll_status ll_sink_window_attn_unrotated(ll_cache* cache, int layer, const void* q, void* out, void* stream) {
    CHECK_CACHE_LAYER(cache, layer);
    if (!cache->dev) return fail(LL_ERR_INVALID_ARG, "index-only handle has no device cache");
    if (!q || !out) return fail(LL_ERR_INVALID_ARG, "null tensor");
    if (!aligned16(q, out)) return fail(LL_ERR_INVALID_ARG, "tensors must be 16-byte aligned");
    const LayerIndex& L = cache->layer[layer];
    if (L.staged_n == 0) return fail(LL_ERR_STATE, "layer %d: no staged chunk", layer);
    std::vector<ChunkWork> work(1);
    work[0].q_begin = 0;
    work[0].q_end = L.staged_n * cache->g.P;
    work[0].ranges = live_ranges(cache->g, L);
    work[0].f0 = L.staged_f0;
    work[0].t_row = cache->staged_t_row[layer];       // where the last cache write left the staged chunk's frames
    if (cache->fmt) return fail(LL_ERR_UNSUPPORTED, "the 8-bit cache takes its queries in ll_chunk_append");
    if (!can_turn_queries(cache, work))
        return fail(LL_ERR_UNSUPPORTED, "unrotated queries need the default kernel and a sink that is not re-indexed for this chunk");
    AttnLaunches launches;
    ll_status st = build_attn(cache, layer, work, q, out, launches, true);
    if (st != LL_OK) return st;
    return launch_built_attn(launches, static_cast<hipStream_t>(stream));
}

// use_static_stage: an 8-bit cache stages its E4M3 queries in the library's own static array instead of the area
// of the caller's cache buffer
static ll_status recache_prefill(ll_cache* cache, int layer, int include_sink, int64_t win_start, int n_win, const void* q,
                                 const void* k, const void* v, void* out, void* stream, bool use_static_stage) {
    CHECK_CACHE_LAYER(cache, layer);
    const Geometry& g = cache->g;
    if (n_win < 0 || n_win > g.ring()) return fail(LL_ERR_INVALID_ARG, "n_win %d outside [0, %d]", n_win, g.ring());
    if (win_start < g.S) return fail(LL_ERR_INVALID_ARG, "win_start %lld overlaps the sink [0, %d)", (long long)win_start, g.S);
    const int n_total = (include_sink ? g.S : 0) + n_win;
    if (n_total == 0) return fail(LL_ERR_INVALID_ARG, "no frames to prefill");
    if (n_win == 0 && win_start != g.S)
        return fail(LL_ERR_INVALID_ARG, "n_win 0 (the sink alone) needs win_start == %d: the next chunk follows the sink", g.S);
    const bool any_null = !q || !k || !v || !out;
    if (cache->dev && any_null) return fail(LL_ERR_INVALID_ARG, "null tensor");
    if (!cache->dev && !(!q && !k && !v && !out)) return fail(LL_ERR_INVALID_ARG, "index-only handle takes null tensors");
    if (cache->dev && (out == q || out == k || out == v)) return fail(LL_ERR_INVALID_ARG, "out must not alias q, k or v");
    if (!aligned16(q, k, v, out)) return fail(LL_ERR_INVALID_ARG, "tensors must be 16-byte aligned");
    LayerIndex& L = cache->layer[layer];
    if (!include_sink && L.sink_have < g.S) return fail(LL_ERR_STATE, "layer %d: sink incomplete (%lld of %d frames)", layer, (long long)L.sink_have, g.S);
    // the bookkeeping is advanced on a copy and the launches are prepared (every check made) before anything is
    // enqueued: a request that cannot run leaves the layer as it was
    const std::vector<ChunkSpan> chunks = prefill_chunks(g, include_sink != 0, win_start, n_win);
    LayerIndex next = L;
    begin_prefill(g, next, include_sink != 0, win_start);
    std::vector<ChunkWork> work;
    int row = 0;
    for (const ChunkSpan& c : chunks) {
        prefill_stage(g, next, c.f0, c.n);
        ChunkWork w;
        w.q_begin = row; w.q_end = row + c.n * g.P;
        w.ranges = live_ranges(g, next);
        w.f0 = c.f0;
        w.t_row = row / g.P;                          // frames of the call, in row order
        work.push_back(w);
        row = w.q_end;
    }
    if (!cache->dev) { L = next; return LL_OK; }
    // rotated queries are staged in `out`; the attention kernel reads and overwrites them in place (bf16: a
    // wave reads exactly the rows it writes).  E4M3 queries are half as wide as the output rows, so they are
    // staged in the cache buffer's own area instead.
    void* q_stage = cache->fmt ? static_cast<void*>(cache->q8_stage) : out;
    // bf16 cache, default kernel: the attention kernel turns the queries as it loads them, the cache write takes keys
    // and values only and the rotated queries never go through memory
    const bool turn_in_attn = can_turn_queries(cache, work);
    ll_status st = LL_OK;
    if (cache->fmt && use_static_stage) {
        const size_t need = size_t(n_total) * g.P * cache->H * cache->D;      // one byte per element
        if (need > STATIC_STAGE_BYTES)
            return fail(LL_ERR_BUFFER_TOO_SMALL, "the re-prefill stages %zu bytes of queries, the static area holds %zu", need, STATIC_STAGE_BYTES);
        st = static_stage(&q_stage);
        if (st != LL_OK) return st;
    }
    AttnLaunches launches;
    st = turn_in_attn ? build_attn(cache, layer, work, q, out, launches, true)
                      : build_attn(cache, layer, work, q_stage, out, launches);
    if (st != LL_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    std::vector<int64_t> frames;
    for (const ChunkSpan& c : chunks)
        for (int i = 0; i < c.n; ++i) frames.push_back(c.f0 + i);
    st = turn_in_attn ? enqueue_append(cache, layer, frames.data(), int(frames.size()), nullptr, k, v, nullptr, s)
                      : enqueue_append(cache, layer, frames.data(), int(frames.size()), q, k, v, q_stage, s);
    if (st == LL_OK) st = launch_built_attn(launches, s);
    // a launch that failed half way leaves slots overwritten that the old bookkeeping still describes: forget the
    // layer, so that later calls report LL_ERR_STATE instead of reading a half-written cache
    L = st == LL_OK ? next : LayerIndex();
    cache->staged_t_row[layer] = work.empty() ? 0 : work.back().t_row;
    return st;
}

ll_status ll_recache_prefill(ll_cache* cache, int layer, int include_sink, int64_t win_start, int n_win, const void* q,
                             const void* k, const void* v, void* out, void* stream) {
    return recache_prefill(cache, layer, include_sink, win_start, n_win, q, k, v, out, stream, false);
}

ll_status ll_recache_prefill_static(ll_cache* cache, int layer, int include_sink, int64_t win_start, int n_win,
                                    const void* q, const void* k, const void* v, void* out, void* stream) {
    return recache_prefill(cache, layer, include_sink, win_start, n_win, q, k, v, out, stream, true);
}

ll_status ll_cache_live_frames(const ll_cache* cache, int layer, int64_t* frames, int cap, int* n) {
    CHECK_CACHE_LAYER(cache, layer);
    if (!n) return fail(LL_ERR_INVALID_ARG, "n is null");
    const std::vector<int64_t> f = live_frames(cache->g, cache->layer[layer]);
    *n = int(f.size());
    if (int(f.size()) > cap || (!frames && !f.empty())) return fail(LL_ERR_BUFFER_TOO_SMALL, "%zu frames, capacity %d", f.size(), cap);
    for (size_t i = 0; i < f.size(); ++i) frames[i] = f[i];
    return LL_OK;
}

ll_status ll_cache_slot_of_frame(const ll_cache* cache, int layer, int64_t frame, int64_t* token_slot) {
    CHECK_CACHE_LAYER(cache, layer);
    if (!token_slot) return fail(LL_ERR_INVALID_ARG, "token_slot is null");
    if (frame < 0) return fail(LL_ERR_INVALID_ARG, "negative frame");
    *token_slot = slot_of_frame(cache->g, frame);
    return LL_OK;
}

ll_status ll_cache_live_ranges(const ll_cache* cache, int layer, int64_t* ranges, int cap, int* n) {
    CHECK_CACHE_LAYER(cache, layer);
    if (!n) return fail(LL_ERR_INVALID_ARG, "n is null");
    const std::vector<SlotRange> r = live_ranges(cache->g, cache->layer[layer]);
    *n = int(r.size());
    if (int(r.size()) > cap || (!ranges && !r.empty())) return fail(LL_ERR_BUFFER_TOO_SMALL, "%zu ranges, capacity %d", r.size(), cap);
    for (size_t i = 0; i < r.size(); ++i) { ranges[2 * i] = r[i].begin; ranges[2 * i + 1] = r[i].end; }
    return LL_OK;
}

ll_status ll_cache_read_frame(const ll_cache* cache, int layer, int64_t frame, void* k_out, void* v_out, void* stream) {
    CHECK_CACHE_LAYER(cache, layer);
    if (!k_out && !v_out) return fail(LL_ERR_INVALID_ARG, "k_out and v_out are both null");
    if (!aligned16(k_out, v_out)) return fail(LL_ERR_INVALID_ARG, "tensors must be 16-byte aligned");
    if (!cache->dev) return fail(LL_ERR_INVALID_ARG, "index-only handle has no device cache");
    if (!frame_held(cache->g, cache->layer[layer], frame)) return fail(LL_ERR_STATE, "layer %d does not hold frame %lld", layer, (long long)frame);
    ReadFrameParams p{};
    p.head_stride = cache->head_stride;
    if (cache->fmt) {
        p.k8_cache = layer_k8(cache, layer); p.v8_cache = layer_v8(cache, layer);
        p.k8_out = static_cast<uint8_t*>(k_out); p.v8_out = static_cast<uint8_t*>(v_out);
    } else {
        p.k_cache = layer_k(cache, layer); p.v_cache = layer_v(cache, layer);
        p.k_out = static_cast<uint16_t*>(k_out); p.v_out = static_cast<uint16_t*>(v_out);
    }
    p.H = cache->H; p.D = cache->D; p.P = cache->g.P; p.slot = slot_of_frame(cache->g, frame);
    hipError_t e = cache->fmt ? launch_read_frame8(p, static_cast<hipStream_t>(stream)) : launch_read_frame(p, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e, "read_frame kernel launch");
    return LL_OK;
}

ll_status ll_cache_set_sink_relative(ll_cache* cache, int on) {
    if (!cache) return fail(LL_ERR_INVALID_ARG, "cache is null");
    if (on && cache->fmt) return fail(LL_ERR_UNSUPPORTED, "the 8-bit cache has no sink-relative mode");
    cache->sink_relative = on != 0;
    return LL_OK;
}

const char* ll_status_string(ll_status s) {
    switch (s) {
        case LL_OK: return "LL_OK";
        case LL_ERR_INVALID_ARG: return "LL_ERR_INVALID_ARG";
        case LL_ERR_STATE: return "LL_ERR_STATE";
        case LL_ERR_BUFFER_TOO_SMALL: return "LL_ERR_BUFFER_TOO_SMALL";
        case LL_ERR_UNSUPPORTED: return "LL_ERR_UNSUPPORTED";
        case LL_ERR_HIP: return "LL_ERR_HIP";
    }
    return "LL_ERR_?";
}
const char* ll_last_error(void) { return g_err.c_str(); }

}  // extern "C"

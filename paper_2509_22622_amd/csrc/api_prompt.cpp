// C-ABI, prompt side of KV-recache (include/longlive.h: ll_prompt_*, ll_cross_attn): host bookkeeping and launches.
#include "api_common.h"

using namespace ll;
using namespace ll_api;

extern "C" {

// ---- the prompt side: per-layer keys and values of the active prompt, in the bf16 cache's kblock layout
struct ll_prompt {
    int layers, H, D, max_tokens;
    char* dev;                  // null for an index-only handle
    int64_t kblocks;            // kblocks per head region (with the readable padding)
    int64_t head_stride;        // elements between heads (K region + V region)
    int64_t layer_stride;
    const double* zero_freq;    // D/2 zeros: the append kernel's rotary step with these turns nothing
    std::vector<int> tokens;    // current prompt length per layer
};

namespace {
struct PromptSizes { int64_t kblocks, head_stride, layer_stride; size_t table_off, total; };
constexpr int MAX_PROMPT_TOKENS = 1 << 16;
bool prompt_shapes_ok(int layers, int H, int D, int max_tokens) {
    return layers >= 1 && H >= 1 && (D == 64 || D == 128) && max_tokens >= 1 && max_tokens <= MAX_PROMPT_TOKENS &&
           int64_t(layers) * H < (int64_t(1) << 24);
}
PromptSizes prompt_sizes(int layers, int H, int D, int max_tokens) {
    PromptSizes z{};
    z.kblocks = (max_tokens + KBLOCK - 1) / KBLOCK + PAD_KBLOCKS;
    z.head_stride = 2 * z.kblocks * KBLOCK * D;
    z.layer_stride = z.head_stride * H;
    z.table_off = (size_t(z.layer_stride) * layers * 2 + 255) & ~size_t(255);
    z.total = (z.table_off + size_t(D / 2) * sizeof(double) + 255) & ~size_t(255);
    return z;
}
}  // namespace

size_t ll_prompt_bytes(int layers, int heads, int head_dim, int max_tokens) {
    if (!prompt_shapes_ok(layers, heads, head_dim, max_tokens)) return 0;
    return prompt_sizes(layers, heads, head_dim, max_tokens).total;
}

ll_status ll_prompt_create(int layers, int heads, int head_dim, int max_tokens, void* dev_buffer, size_t dev_bytes,
                           ll_prompt** out) {
    if (!out) return fail(LL_ERR_INVALID_ARG, "out is null");
    *out = nullptr;
    if (!prompt_shapes_ok(layers, heads, head_dim, max_tokens))
        return fail(head_dim != 64 && head_dim != 128 && head_dim > 0 ? LL_ERR_UNSUPPORTED : LL_ERR_INVALID_ARG,
                    "bad shape: layers %d heads %d head_dim %d (64 or 128) max_tokens %d (1..%d)", layers, heads,
                    head_dim, max_tokens, MAX_PROMPT_TOKENS);
    const bool index_only = dev_buffer == nullptr && dev_bytes == 0;
    const PromptSizes z = prompt_sizes(layers, heads, head_dim, max_tokens);
    if (!index_only) {
        if (!dev_buffer) return fail(LL_ERR_INVALID_ARG, "dev_buffer is null");
        if (reinterpret_cast<uintptr_t>(dev_buffer) & 255) return fail(LL_ERR_INVALID_ARG, "dev_buffer is not 256-byte aligned");
        if (dev_bytes < z.total) return fail(LL_ERR_BUFFER_TOO_SMALL, "dev_buffer has %zu bytes, %zu needed", dev_bytes, z.total);
        hipError_t e = hipMemset(dev_buffer, 0, z.total);
        if (e == hipSuccess) e = hipDeviceSynchronize();
        if (e != hipSuccess) return hip_fail(e, "ll_prompt_create: clearing the buffer");
    }
    ll_prompt* pr = new ll_prompt();
    pr->layers = layers; pr->H = heads; pr->D = head_dim; pr->max_tokens = max_tokens;
    pr->dev = static_cast<char*>(dev_buffer);
    pr->kblocks = z.kblocks; pr->head_stride = z.head_stride; pr->layer_stride = z.layer_stride;
    pr->zero_freq = index_only ? nullptr : reinterpret_cast<const double*>(pr->dev + z.table_off);
    pr->tokens.assign(layers, 0);
    *out = pr;
    return LL_OK;
}

ll_status ll_prompt_destroy(ll_prompt* prompt) {
    delete prompt;
    return LL_OK;
}

#define CHECK_PROMPT_LAYER(prompt, layer)                                           \
    if (!(prompt)) return fail(LL_ERR_INVALID_ARG, "prompt is null");               \
    if ((layer) < 0 || (layer) >= (prompt)->layers)                                 \
        return fail(LL_ERR_INVALID_ARG, "layer %d out of range [0, %d)", (layer), (prompt)->layers)

static uint16_t* prompt_k(const ll_prompt* pr, int layer) {
    return reinterpret_cast<uint16_t*>(pr->dev) + int64_t(layer) * pr->layer_stride;
}
static uint16_t* prompt_v(const ll_prompt* pr, int layer) { return prompt_k(pr, layer) + pr->kblocks * KBLOCK * pr->D; }

ll_status ll_prompt_recache(ll_prompt* prompt, int layer, const void* k, const void* v, int n_tokens, void* stream) {
    CHECK_PROMPT_LAYER(prompt, layer);
    if (n_tokens < 1 || n_tokens > prompt->max_tokens)
        return fail(LL_ERR_INVALID_ARG, "n_tokens %d outside [1, %d]", n_tokens, prompt->max_tokens);
    if (prompt->dev && (!k || !v)) return fail(LL_ERR_INVALID_ARG, "null tensor");
    if (!prompt->dev && (k || v)) return fail(LL_ERR_INVALID_ARG, "index-only handle takes null tensors");
    if (!aligned16(k, v)) return fail(LL_ERR_INVALID_ARG, "tensors must be 16-byte aligned");
    if (prompt->dev) {
        // The cache-write kernel of ll_chunk_append with one "frame" of n_tokens tokens at slot 0, no queries, and
        // its rotary step switched off: the keys pass unchanged bit for bit.
        AppendParams p{};
        p.k = static_cast<const uint16_t*>(k); p.v = static_cast<const uint16_t*>(v);
        p.k_cache = prompt_k(prompt, layer); p.v_cache = prompt_v(prompt, layer);
        p.head_stride = prompt->head_stride;
        p.rope = RopeTables{prompt->zero_freq, nullptr, nullptr, prompt->D / 2, 0, 0};
        p.identity = 1;
        p.H = prompt->H; p.D = prompt->D; p.P = n_tokens; p.grid_w = n_tokens;
        p.n_frames = 1;
        p.frame[0] = 0; p.slot[0] = 0;
        p.seg_begin[0] = 0; p.seg_begin[1] = (n_tokens + KBLOCK - 1) / KBLOCK;
        hipError_t e = launch_append(p, static_cast<hipStream_t>(stream));
        if (e != hipSuccess) return hip_fail(e, "prompt cache-write kernel launch");
    }
    prompt->tokens[layer] = n_tokens;
    return LL_OK;
}

ll_status ll_prompt_tokens(const ll_prompt* prompt, int layer, int* n_tokens) {
    CHECK_PROMPT_LAYER(prompt, layer);
    if (!n_tokens) return fail(LL_ERR_INVALID_ARG, "n_tokens is null");
    *n_tokens = prompt->tokens[layer];
    return LL_OK;
}

// out_frag: the output goes to `out` in the output projection's fragment order instead of row-major
static ll_status cross_attn(const ll_prompt* prompt, int layer, const void* q, int n_q, void* out, bool out_frag, void* stream);

ll_status ll_cross_attn(const ll_prompt* prompt, int layer, const void* q, int n_q, void* out, void* stream) {
    return cross_attn(prompt, layer, q, n_q, out, false, stream);
}

ll_status ll_out_proj_pack_weight(int heads, int head_dim, const void* w_out, void* w_packed, void* stream) {
    if (heads < 1 || heads > 1024 || (head_dim != 64 && head_dim != 128))
        return fail(LL_ERR_INVALID_ARG, "heads %d (1..1024) or head_dim %d (64 or 128)", heads, head_dim);
    if (!w_out || !w_packed) return fail(LL_ERR_INVALID_ARG, "null tensor");
    if (!aligned16(w_out, w_packed)) return fail(LL_ERR_INVALID_ARG, "tensors must be 16-byte aligned");
    if (w_out == w_packed) return fail(LL_ERR_INVALID_ARG, "w_packed must not be w_out");
    const int n = heads * head_dim;
    hipError_t e = launch_pack_out_weight(static_cast<const uint16_t*>(w_out), static_cast<uint16_t*>(w_packed), n, n,
                                          static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e, "weight packing kernel launch");
    return LL_OK;
}

size_t ll_cross_attn_out_workspace_bytes(int heads, int head_dim, int n_q) {
    if (heads < 1 || heads > 1024 || (head_dim != 64 && head_dim != 128) || n_q < 1 || n_q > (1 << 24)) return 0;
    return (size_t(n_q) + 15) / 16 * 16 * size_t(heads) * size_t(head_dim) * 2;
}

ll_status ll_cross_attn_out(const ll_prompt* prompt, int layer, const void* q, int n_q, const void* w_packed,
                            void* workspace, void* y, void* stream) {
    CHECK_PROMPT_LAYER(prompt, layer);
    if (prompt->dev) {
        if (!w_packed || !y) return fail(LL_ERR_INVALID_ARG, "null tensor");
        if (!aligned16(w_packed, y)) return fail(LL_ERR_INVALID_ARG, "tensors must be 16-byte aligned");
        if (y == workspace || y == q || w_packed == workspace || w_packed == y || workspace == q)
            return fail(LL_ERR_INVALID_ARG, "y, w_packed and workspace must not overlap the other tensors");
    } else if (w_packed || y) {
        return fail(LL_ERR_INVALID_ARG, "index-only handle takes null tensors");
    }
    ll_status st = cross_attn(prompt, layer, q, n_q, workspace, true, stream);   // every other check, and the attention
    if (st != LL_OK || !prompt->dev) return st;
    OutProjParams p{};
    p.x_frag = static_cast<const uint16_t*>(workspace); p.w_frag = static_cast<const uint16_t*>(w_packed);
    p.y = static_cast<uint16_t*>(y);
    p.M = n_q; p.N = p.K = prompt->H * prompt->D;
    hipError_t e = launch_out_proj(p, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e, "output projection kernel launch");
    return LL_OK;
}

static ll_status cross_attn(const ll_prompt* prompt, int layer, const void* q, int n_q, void* out, bool out_frag, void* stream) {
    CHECK_PROMPT_LAYER(prompt, layer);
    if (n_q < 1 || n_q > (1 << 24)) return fail(LL_ERR_INVALID_ARG, "n_q %d outside [1, 2^24]", n_q);
    if (prompt->tokens[layer] == 0) return fail(LL_ERR_STATE, "layer %d: no prompt", layer);
    if (!prompt->dev) {
        if (q || out) return fail(LL_ERR_INVALID_ARG, "index-only handle takes null tensors");
        return LL_OK;
    }
    if (!q || !out) return fail(LL_ERR_INVALID_ARG, "null tensor");
    if (!aligned16(q, out)) return fail(LL_ERR_INVALID_ARG, "tensors must be 16-byte aligned");
    // these queries carry no factor yet: only kernels that apply AttnParams::scale_log2e themselves qualify
    // A workgroup meets few kblocks here, and most of its life is the load of its queries and the store of its
    // outputs.  With one round of workgroups on the chip (a chunk's queries) the pipelined kernel is the quicker one;
    // with several rounds (a re-prefill's queries) small workgroups, three to a CU in different phases, are.
    int variant = attn_variant_qscale(prompt->D);
    if ((int64_t(n_q) + 255) / 256 * prompt->H > 512) variant = attn_variant_short_keys(prompt->D);
    if (g_variant != 0 && attn_variant_supports(g_variant, prompt->D, KBLOCK) && attn_variant_applies_scale(g_variant) &&
        (!out_frag || attn_variant_out_frag(g_variant)))
        variant = g_variant;
    AttnParams p{};
    p.q = static_cast<const uint16_t*>(q);
    if (out_frag) p.out_frag = static_cast<uint16_t*>(out);
    else p.out = static_cast<uint16_t*>(out);
    p.k_cache = prompt_k(prompt, layer); p.v_cache = prompt_v(prompt, layer);
    p.head_stride = prompt->head_stride;
    p.H = prompt->H; p.D = prompt->D;
    p.kblock = KBLOCK;
    p.scale_log2e = float(1.4426950408889634 / std::sqrt(double(prompt->D)));
    p.n_chunks = 1;
    AttnChunk& ch = p.chunk[0];
    ch.q_begin = 0; ch.q_end = n_q; ch.tile_begin = 0;
    ch.n_ranges = 1; ch.rs[0] = 0; ch.re[0] = prompt->tokens[layer];
    const int qt = attn_variant_qtile(variant);
    p.n_tiles = (n_q + qt - 1) / qt;
    hipError_t e = launch_attn(p, variant, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e, "cross-attention kernel launch");
    return LL_OK;
}

}  // extern "C"

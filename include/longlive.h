/*
 * longlive.h - C-ABI of the MI355X (gfx950) library for LongLive's inference hot
 * path: short-window attention with a frame-level attention sink over a rolling
 * per-layer KV cache, and the chunk-causal re-prefill used by KV-recache.
 *
 * Paper passages behind each call are named at the call.  Shapes use the
 * paper's names: chunk (C frames), local window (W frames), sink (S frames);
 * P = tokens per frame, H = heads, D = head_dim.
 *
 * Conventions for every call
 *   - Return value is an ll_status; nothing throws or aborts across this ABI.
 *     ll_last_error() gives a thread-local message for the last failure.
 *   - "device" pointers are HIP device memory of the current device, "host"
 *     pointers are ordinary process memory.  Tensors are bfloat16, token-major
 *     [tokens, H, D], densely packed, 16-byte aligned; tokens of a chunk are frame-major
 *     and row-major (y * grid_w + x) inside a frame.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Device
 *     work is enqueued on it and the call returns without synchronising.  Tensors
 *     are borrowed until the stream has passed the call.
 *   - The cache's device buffer is owned by the caller and must outlive the
 *     handle.  The library allocates no device memory.
 *   - Host-side bookkeeping changes at call time, so calls for one layer must be
 *     made in program order; layers are independent of each other.
 *   - One handle = one video (batch 1, the paper's interactive setting).
 */
#ifndef LONGLIVE_H
#define LONGLIVE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ll_cache ll_cache; /* opaque; host bookkeeping only */

typedef enum {
    LL_OK = 0,
    LL_ERR_INVALID_ARG = 1,      /* null pointer, value out of range, shape mismatch      */
    LL_ERR_STATE = 2,            /* call out of order for this layer                       */
    LL_ERR_BUFFER_TOO_SMALL = 3, /* caller's buffer smaller than required                  */
    LL_ERR_UNSUPPORTED = 4,      /* valid request this build has no kernel for             */
    LL_ERR_HIP = 5               /* a HIP runtime call failed (message has the HIP error)  */
} ll_status;

/* Bytes of device memory ll_cache_create needs for these shapes; 0 if they are invalid.
 * Resident size is O(S + W + C) frames per layer and independent of video length
 * (Sec. 3.3, "Consistency between Training and Inference"). */
size_t ll_cache_bytes(int layers, int heads, int head_dim, int tokens_per_frame,
                      int sink_frames, int window_frames, int chunk_frames);

/* Create the bookkeeping for `layers` independent rolling caches laid out in `dev_buffer`.
 *   Key set of a chunk starting at frame f0 (Sec. 3.3 "Frame Sink", "Short-window
 *   Attention"): sink frames [0, S), the last W non-sink frames before f0, and the chunk
 *   itself.  window_frames counts past frames only; the ring holds W + C frames.
 *   head_dim must be 64 or 128; tokens_per_frame must equal grid_h * grid_w;
 *   chunk_frames >= 1, sink_frames >= 0, window_frames >= 0.
 *   rope_theta: base of the rotary embedding (10000 for the benchmark configs).
 *   dev_buffer: device, 256-byte aligned, at least ll_cache_bytes(...) bytes; it is zeroed
 *   and the rotary tables are written into its tail (synchronous copies on the null
 *   stream).  dev_buffer == NULL with dev_bytes == 0 makes an index-only handle: the
 *   bookkeeping and the introspection calls work, compute calls accept NULL tensors and
 *   enqueue nothing (used to test the indexing without a GPU). */
ll_status ll_cache_create(int layers, int heads, int head_dim, int tokens_per_frame,
                          int sink_frames, int window_frames, int chunk_frames,
                          int grid_h, int grid_w, float rope_theta,
                          void* dev_buffer, size_t dev_bytes, ll_cache** out);

/* The 8-bit variant of the cache: rotated keys, values and rotated queries are held as 8-bit floating point
 * numbers (OCP E4M3: 4 exponent bits with bias 7, 3 mantissa bits, largest value 448) and both products of the
 * attention run on the fp8 matrix instructions.  The paper quantises the model's weights to 8 bits and reports
 * that quality holds (Appendix "Quantization" and its table); applying 8 bits to the attention operands is this
 * library's extension, with its own, looser accuracy: the result differs from ll_cache_create's by a few per cent
 * in relative L2 norm on random inputs.  Everything else is as for ll_cache_create, and every call below takes
 * either kind of handle.  Definition (e4m3 = nearest E4M3 value, ties to even, |x| clamped to 448 first):
 *     K8 = e4m3(K' * 2^-k_exp), V8 = e4m3(V * 2^-v_exp), Q8 = e4m3(q' * log2(e)/sqrt(D) * 2^k_exp),
 *     out = 2^v_exp * sum_j w_j V8_j / sum_j w_j,   w_j = 2^(Q8 . K8_j - max);
 *   the kernel also rounds the weights w_j to E4M3 (relative to a running reference) before the second product.
 *   k_exp, v_exp in [-16, 16]: powers of two (exact to apply) that bring K' and V into E4M3's range; 0 suits
 *   inputs of magnitude up to a few hundred, and a floating point format needs no finer (per-frame) scale.
 *   Differences for the other calls with such a handle:
 *     - q_out of ll_chunk_append and q_roped of ll_sink_window_attn are [n*P, H, D] bytes (E4M3 codes);
 *       q_out must not alias q.  q, k, v and out stay bfloat16.
 *     - ll_recache_prefill stages its queries in an area of the cache buffer shared by all layers: two prefill
 *       calls on one handle must not overlap in time (enqueue them on one stream).  out is written only.
 *     - ll_cache_read_frame returns codes: k_out, v_out are [P, H, D] bytes.
 *   ll_cache_bytes_fp8 gives the buffer size (about half of ll_cache_bytes plus the staging area). */
size_t ll_cache_bytes_fp8(int layers, int heads, int head_dim, int tokens_per_frame,
                          int sink_frames, int window_frames, int chunk_frames);
ll_status ll_cache_create_fp8(int layers, int heads, int head_dim, int tokens_per_frame,
                              int sink_frames, int window_frames, int chunk_frames,
                              int grid_h, int grid_w, float rope_theta, int k_exp, int v_exp,
                              void* dev_buffer, size_t dev_bytes, ll_cache** out);

/* Free the host bookkeeping.  The device buffer stays with the caller. */
ll_status ll_cache_destroy(ll_cache* cache);

/* Forget every frame of `layer` (-1 = all layers): the next append must start at frame 0. */
ll_status ll_cache_reset(ll_cache* cache, int layer);

/* Stage chunk [frame_start, frame_start + n_frames) of `layer`  (Appendix Alg. 2: every
 * denoising pass of a chunk runs with the chunk's own K/V, only the final clean pass stays).
 *   Rotates q and k by the 3D rotary embedding at (absolute frame, row, column) in fp32,
 *   writes q_out = bf16(rotated q * log2(e)/sqrt(D)) (the softmax scale is folded in here, with
 *   one rounding; q_out may alias q) and rotated k and v into the layer's cache slots.
 *   frame_start equal to the staged chunk's start  -> overwrite the same slots;
 *   frame_start equal to staged start + its length -> the staged chunk becomes permanent,
 *       frames older than frame_start - W (non-sink) stop being live, sink frames stay;
 *   first call after create/reset must have frame_start 0; anything else -> LL_ERR_STATE.
 *   1 <= n_frames <= chunk_frames.  q, k, v, q_out: device, [n_frames*P, H, D] bf16.
 *   q and q_out may both be NULL (bf16 cache): keys and values only; the chunk's queries then go, unrotated, to
 *   ll_sink_window_attn_unrotated, and the rotated queries never pass through memory. */
ll_status ll_chunk_append(ll_cache* cache, int layer, int64_t frame_start, int n_frames,
                          const void* q, const void* k, const void* v, void* q_out,
                          void* stream);

/* out = softmax(q_roped K^T / sqrt(D)) V over sink U window U staged chunk of `layer`
 * (Sec. 3.3; no mask inside the key set: bidirectional within the chunk, the rest is past).
 *   q_roped: device, [Nq, H, D] bf16, the (pre-scaled) q_out of the matching ll_chunk_append, where
 *   Nq = staged n_frames * P.  out: device, same shape (may alias q_roped).
 *   LL_ERR_STATE if no chunk is staged. */
ll_status ll_sink_window_attn(ll_cache* cache, int layer, const void* q_roped, void* out,
                              void* stream);
/* The same attention (Sec. 3.3) from the queries as the model's projection made them: q: device, [Nq, H, D] bf16,
 * unrotated and unscaled, the rows of the staged chunk's frames in order.  The kernel applies the 3D rotary
 * embedding at each row's (absolute frame, row, column) and the factor log2(e)/sqrt(D) as it loads the queries, with
 * the arithmetic and the one rounding of ll_chunk_append's q_out, so the result is bit for bit that of
 * ll_chunk_append(q, q_out) followed by ll_sink_window_attn(q_out).  The chunk must have been staged by
 * ll_chunk_append (with or without queries) or ll_recache_prefill on the same stream before.  out must not alias q.
 * bf16 cache only (LL_ERR_UNSUPPORTED for an 8-bit cache, for a chunk whose sink is re-indexed by
 * ll_cache_set_sink_relative, and while a diagnostic kernel variant is forced); other errors as above. */
ll_status ll_sink_window_attn_unrotated(ll_cache* cache, int layer, const void* q, void* out, void* stream);

/* KV-recache for one layer (Sec. 3.1 "KV Recache"; Sec. 3.3 last sentence; Alg. 2 line
 * "recache"): rebuild the cache from frames [0, S) (if include_sink) followed by
 * [win_start, win_start + n_win), and compute their attention under the chunk-causal mask:
 * the frames are cut into chunks of C (the sink first, then the window from win_start);
 * a chunk starting at f0 sees the sink, the retained frames in [f0 - W, f0) and itself.
 *   q, k, v, out: device, [(S if include_sink else 0) + n_win) * P, H, D] bf16 in that
 *   frame order.  out receives the attention output; it must not alias q, k or v (the attention kernel reads q while
 *   other rows of out are written; where the kernel cannot turn the queries itself - a forced diagnostic variant, a
 *   re-indexed sink - out also serves as the staging area for the rotated queries).
 *   All non-sink frames held before are dropped.  include_sink == 0 keeps the sink K/V
 *   already held (LL_ERR_STATE if the sink is incomplete).  win_start >= S, 0 <= n_win <=
 *   W + C; n_win == 0 (the sink alone, include_sink != 0) requires win_start == S.
 *   Afterwards the layer is as if those frames had been streamed: the last chunk
 *   is staged and the next ll_chunk_append must start at win_start + n_win (or repeat the
 *   last chunk's start).  Every check is made before anything is enqueued: a refused call leaves
 *   the layer untouched.  If a kernel launch itself fails (LL_ERR_HIP) the layer's slots may be
 *   half rewritten: the layer is then reset (as by ll_cache_reset), later calls on it return
 *   LL_ERR_STATE until it is filled again from frame 0 or by another re-prefill with the sink. */
ll_status ll_recache_prefill(ll_cache* cache, int layer, int include_sink, int64_t win_start,
                             int n_win, const void* q, const void* k, const void* v,
                             void* out, void* stream);

/* ll_recache_prefill for callers that must not allocate or hand over scratch memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): same arguments, same result, and no device memory beyond
 * the inputs, the outputs and the cache itself is taken from the caller.  The one scratch buffer the re-prefill
 * needs - the E4M3 queries of an 8-bit cache, which ll_recache_prefill stages in an area of the cache buffer -
 * lives in an array inside the library instead: 36 MiB per GPU the library is used on, held until the process
 * ends (a re-prefill of 15 frames at 1560 tokens x 12 heads x 128 needs 34.3 MiB).
 *   LL_ERR_BUFFER_TOO_SMALL if (frames to prefill) * P * H * D exceeds 36 MiB (nothing is enqueued).
 *   Every call on one GPU shares that GPU's array: two such calls must not overlap in time on one GPU, whatever
 *   their handles or layers (enqueue them on one stream, or order the streams); the array keeps the last call's
 *   queries, nothing in it needs clearing (every byte a call reads it has written before).
 *   A bf16 cache needs no scratch (its queries are turned by the attention kernel as it loads them, or staged in
 *   `out`): for such a handle the call is ll_recache_prefill.  Neither call allocates, frees or synchronises. */
ll_status ll_recache_prefill_static(ll_cache* cache, int layer, int include_sink, int64_t win_start,
                                    int n_win, const void* q, const void* k, const void* v,
                                    void* out, void* stream);

/* ---- introspection (exact integer answers; used for the bit-exact indexing checks) ---- */

/* Frames the staged chunk attends to, ascending.  frames: host, capacity `cap`; *n = count. */
ll_status ll_cache_live_frames(const ll_cache* cache, int layer, int64_t* frames, int cap,
                               int* n);
/* First token slot of `frame` in the per-head key order: f*P for a sink frame, else
 * (S + (f - S) mod (W + C)) * P. */
ll_status ll_cache_slot_of_frame(const ll_cache* cache, int layer, int64_t frame,
                                 int64_t* token_slot);
/* The staged chunk's key set as at most 3 half-open token-slot ranges, ascending and
 * disjoint.  ranges: host int64[2*cap] as (begin, end) pairs; *n = count. */
ll_status ll_cache_live_ranges(const ll_cache* cache, int layer, int64_t* ranges, int cap,
                               int* n);
/* Copy one held frame's rotated K and V out of the cache into [P, H, D] bf16 device
 * tensors (either may be NULL, not both: LL_ERR_INVALID_ARG).  LL_ERR_STATE if the frame is not held. */
ll_status ll_cache_read_frame(const ll_cache* cache, int layer, int64_t frame, void* k_out,
                              void* v_out, void* stream);

/* Variant of the rule for very long videos (this library's reading; the paper keeps the first frames as a sink for
 * videos of any length, Sec. 3.3 "Frame Sink", and does not say which rotary positions they get): with absolute
 * frame positions the rotary distance between a query and the sink grows with the video without bound.  With
 * on != 0, every later ll_sink_window_attn and ll_recache_prefill of this handle takes the scores of the sink
 * keys as if the query's frame index were smaller by max(0, f0 - W - S), f0 = first frame of the query's chunk:
 * seen from the queries the sink sits at frames 0 .. S-1 and the oldest window frame at S, wherever in the video
 * the window lies.  Only the frame axis of the rotary embedding is concerned, the other scores are unchanged, and
 * nothing differs while f0 <= W + S.  The cache contents do not depend on the setting (keys stay rotated at their
 * absolute frames; the kernel turns the queries instead, with one more rounding to bfloat16 for the sink's
 * scores).  LL_ERR_UNSUPPORTED for handles of the 8-bit cache; a later attention call returns LL_ERR_UNSUPPORTED
 * if a kernel variant without this mode was selected with ll_set_attn_variant. */
ll_status ll_cache_set_sink_relative(ll_cache* cache, int on);

/* ---- The prompt side of KV-recache (Sec. 3.1 "KV Recache", Fig. 2 right).  The prompt reaches the video tokens
 * through the cross-attention layers; at a prompt switch the cached state is rebuilt from the generated frames paired
 * with the NEW prompt: ll_recache_prefill rebuilds the self-attention side, and the calls below hold, replace and
 * read the per-layer keys and values projected from the prompt's embeddings (the projections belong to the model;
 * k and v come in as tensors).  No mask and no positional embedding: every query sees every prompt token,
 *     out = softmax(q k^T / sqrt(D)) v   per head.
 * A handle is independent of any ll_cache.  Calls for one layer must be made in program order. */
typedef struct ll_prompt ll_prompt;

/* Bytes of device memory ll_prompt_create needs; 0 if the shapes are invalid (head_dim 64 or 128, max_tokens in
 * [1, 65536]). */
size_t ll_prompt_bytes(int layers, int heads, int head_dim, int max_tokens);
/* dev_buffer: device, 256-byte aligned, at least ll_prompt_bytes(...) bytes, owned by the caller, must outlive the
 * handle; it is zeroed (synchronous, null stream).  NULL with dev_bytes == 0 makes an index-only handle whose
 * compute calls take NULL tensors and enqueue nothing. */
ll_status ll_prompt_create(int layers, int heads, int head_dim, int max_tokens, void* dev_buffer, size_t dev_bytes,
                           ll_prompt** out);
ll_status ll_prompt_destroy(ll_prompt* prompt);
/* Replace layer `layer`'s prompt keys and values by those of a (new) prompt of n_tokens tokens, 1 <= n_tokens <=
 * max_tokens.  k, v: device, bf16 [n_tokens, H, D].  Nothing of the former prompt remains visible, also when the new
 * one is shorter.  Enqueues one kernel; later ll_cross_attn calls on the same stream read the new prompt. */
ll_status ll_prompt_recache(ll_prompt* prompt, int layer, const void* k, const void* v, int n_tokens, void* stream);
/* Tokens of layer `layer`'s current prompt (0 before the first ll_prompt_recache). */
ll_status ll_prompt_tokens(const ll_prompt* prompt, int layer, int* n_tokens);
/* Cross-attention of n_q query rows over layer `layer`'s prompt.  q: device, bf16 [n_q, H, D], as the model's query
 * projection made them (the factor log2(e)/sqrt(D) is applied inside the kernel: to the queries, with one rounding of
 * the product to bf16, or to the fp32 scores, depending on the kernel the launch's size selects);
 * out: device, bf16 [n_q, H, D]; out may be q itself (a wave reads exactly the rows it writes), any other overlap is
 * an error the library cannot detect.  1 <= n_q <= 2^24.  LL_ERR_STATE if the layer has no prompt yet. */
ll_status ll_cross_attn(const ll_prompt* prompt, int layer, const void* q, int n_q, void* out, void* stream);
/* The cross-attention block's whole output path (Sec. 3.1, Fig. 2 right): the attention of ll_cross_attn followed by
 * the layer's output projection, y = concat_heads(attn_out) w_out^T, on the same stream.  The two kernels hand the
 * attention output over in the order the matrix instructions of the projection read it (blocks of 16 rows x 32
 * features), not as a row-major tensor; the weight is brought into the same order once, by ll_out_proj_pack_weight.
 *
 * ll_out_proj_pack_weight: w_out: device, bf16 [H*D, H*D] as a linear layer stores its weight ([output feature][input
 *   feature]); w_packed: device, the same number of bytes, 16-byte aligned, must not overlap w_out.  One kernel; done
 *   once per layer when the model is loaded.  head_dim 64 or 128, heads >= 1.  No bias anywhere (an addition the
 *   caller can fuse elsewhere).
 * ll_cross_attn_out_workspace_bytes: bytes of `workspace` for n_q rows (n_q rounded up to 16, x H*D x 2); 0 if a
 *   size is invalid.
 * ll_cross_attn_out: w_packed as written by ll_out_proj_pack_weight for this handle's heads and head_dim (borrowed);
 *   workspace: device, 16-byte aligned, at least ll_cross_attn_out_workspace_bytes(...) bytes, owned by the caller:
 *   receives the attention output in the projection's order and is read again by the projection (its contents
 *   afterwards are that intermediate, of no use to the caller; callers that want the attention output itself use
 *   ll_cross_attn).  y: device, bf16 [n_q, H*D], fp32 accumulation, one rounding.  y, w_packed and workspace must not
 *   overlap one another or q.  Other arguments and errors as for ll_cross_attn. */
ll_status ll_out_proj_pack_weight(int heads, int head_dim, const void* w_out, void* w_packed, void* stream);
size_t ll_cross_attn_out_workspace_bytes(int heads, int head_dim, int n_q);
ll_status ll_cross_attn_out(const ll_prompt* prompt, int layer, const void* q, int n_q, const void* w_packed,
                            void* workspace, void* y, void* stream);

/* ---- The train-time rule and its backward pass (Sec. 3.2 streaming long tuning; Sec. 3.3 "Consistency between
 * Training and Inference").  One training step supervises a clip of n_clip frames that follows the frames generated
 * so far.  Resident keys and values: the S sink frames, the last n_ctx <= W frames of the preceding context (constants:
 * no gradient), and the clip's own frames (with gradient).  The clip is processed chunk by chunk under the inference
 * rule: the chunk starting at frame f0 attends to the sink, to the frames within W before f0 (context or clip) and to
 * itself.  ll_clip_forward computes that attention; ll_clip_backward the gradients of sum(out * dout) with respect
 * to the clip's own q, k and v (before the rotary embedding), in bf16:
 *     P = softmax(q' K'^T / sqrt(D)),  dV = P^T dO,  dZ = P * (dO V^T - rowsum(dO * O)),
 *     dq' = dZ K' / sqrt(D),  dK' = dZ^T q' / sqrt(D),  then back through the rotary turn of each pair.
 * One handle serves one layer at a time: the backward pass differentiates the handle's last forward pass.  All
 * intermediate tensors live in the caller's buffer; nothing is allocated.  The kernels multiply rows of that buffer
 * which lie outside a step's key set by an exact zero instead of clearing them, so the buffer must hold finite
 * numbers only: it is zeroed at ll_clip_create, and q, k, v, dout must be finite in every step (a NaN or an infinity
 * in one step's inputs stays in the buffer and can reach later steps of the same handle). */
typedef struct ll_clip ll_clip;

/* Bytes of device memory ll_clip_create needs; 0 if the shapes are invalid.  clip_frames is the largest n_clip. */
size_t ll_clip_bytes(int heads, int head_dim, int tokens_per_frame, int sink_frames, int window_frames,
                     int clip_frames, int chunk_frames);
/* Arguments as for ll_cache_create (one layer).  dev_buffer: device, 256-byte aligned, at least ll_clip_bytes(...)
 * bytes, zeroed here (synchronous, null stream); NULL with dev_bytes == 0 makes an index-only handle. */
ll_status ll_clip_create(int heads, int head_dim, int tokens_per_frame, int sink_frames, int window_frames,
                         int clip_frames, int chunk_frames, int grid_h, int grid_w, float rope_theta,
                         void* dev_buffer, size_t dev_bytes, ll_clip** out);
ll_status ll_clip_destroy(ll_clip* clip);
/* Forward.  The context is frames [ctx_start, ctx_start + n_ctx), 0 <= n_ctx <= window_frames, the clip the n_clip
 * frames after it.  ctx_start >= sink_frames, or ctx_start == 0 with n_ctx == 0 for a video's first clip, which
 * contains the sink frames itself (they then receive gradients like any clip frame).
 *   q: device bf16 [n_clip * P, H, D], the clip's queries.
 *   k, v: device bf16 [n_frames * P, H, D] for all resident frames in ascending order: the sink frames (unless they
 *         belong to the clip), the context, the clip; all before the rotary embedding.
 *   out: device bf16 [n_clip * P, H, D].  All four tensors are used by the forward pass only: what the backward pass
 *   needs of them (rotated operands, row sums, and the output before its rounding to bf16, from which it takes
 *   delta_i = dO_i . O_i) is kept in the handle's buffer. */
ll_status ll_clip_forward(ll_clip* clip, int64_t ctx_start, int n_ctx, int n_clip, const void* q, const void* k,
                          const void* v, void* out, void* stream);
/* Introspection (works on index-only handles): the key set of chunk `chunk` (0-based, in clip order) of the handle's
 * last forward as at most 2 half-open token-slot ranges into the list of resident frames (sink frames outside the
 * clip, context, clip; P slots per frame), ascending and disjoint.  ranges: host int64[2*cap]; *n = count.
 * LL_ERR_STATE without a forward pass. */
ll_status ll_clip_chunk_key_ranges(const ll_clip* clip, int chunk, int64_t* ranges, int cap, int* n);

/* Backward of the handle's last forward.  dout: device bf16 [n_clip * P, H, D]; dq, dk, dv: device bf16
 * [n_clip * P, H, D], gradients for the clip's own frames (context and sink frames outside the clip are constants).
 * LL_ERR_STATE without a forward pass. */
ll_status ll_clip_backward(ll_clip* clip, const void* dout, void* dq, void* dk, void* dv, void* stream);

const char* ll_status_string(ll_status s);
const char* ll_last_error(void); /* thread-local, never NULL */

#ifdef __cplusplus
}
#endif
#endif /* LONGLIVE_H */

"""Benchmark of the sink+window attention hot path on one MI355X.

A step is one pass of the hot path over one 3-frame chunk: for each of the 30 layers,
ll_chunk_append (rotary + ring write of the keys and values) then ll_sink_window_attn_unrotated (the attention
kernel turns the queries as it loads them; --two-call-step: the rotated queries go through memory and
ll_sink_window_attn reads them), at the Wan-1.3B shape
(12 heads x 128, 1560 tokens/frame, sink 3, window 9, chunk 3: 4680 queries x 23400
keys per layer) in steady state (ring full, wrapping).  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2516.6      # MI355X dense bf16 MFMA: 256 CU x 4096 flop/clk x 2.4 GHz
PEAK_HBM_GBS = 8000.0
# HBM bytes per attention launch: a constant recorded from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this
# workload (profiles/attn_wan_layer_pmc.txt), not measured by the run that prints it:
# fetch 100941 KiB x 2.0 (scale from a device copy of known size in the same run) + write 14042 KiB x 1.0
ATTN_HBM_TRAFFIC_BYTES = int(100941 * 1024 * 2.0 + 14042 * 1024 * 1.0)
ATTN_HBM_TRAFFIC_SOURCE = "profiles/attn_wan_layer_pmc.txt (recorded constant: 1.28 x the algorithmic bytes, 16 (head, XCD) K/V streams for 12 heads)"


def attn_flops(nq, nk, d, h):
    return 4.0 * nq * nk * d * h


def cpu_baseline(w, chunks=3):
    """Time the fp64 oracle as it stands on a bounded sample of the same workload: one layer in steady state,
    all heads, every query row, `chunks` consecutive chunks (append + key-set build + attention each)."""
    from oracle.longlive_oracle import Oracle, OracleConfig
    from paper_2509_22622_amd import synth
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
    o = Oracle(OracleConfig(1, w.heads, w.head_dim, w.grid_h, w.grid_w, w.chunk_frames, w.sink_frames, w.window_frames))
    n_fill = (w.sink_frames + w.window_frames) // w.chunk_frames
    for i in range(n_fill):
        o.append(0, i * w.chunk_frames, *synth.chunk_qkv(w, 0, i))
    t_append = t_attn = 0.0
    for i in range(n_fill, n_fill + chunks):
        q, k, v = synth.chunk_qkv(w, 0, i)
        t0 = time.perf_counter()
        o.append(0, i * w.chunk_frames, q, k, v)
        t1 = time.perf_counter()
        o.attn(0)
        t_attn += time.perf_counter() - t1
        t_append += t1 - t0
        nk = len(o.live_frames(0)) * w.tokens_per_frame
        com = o.layer[0].committed                       # frames the key-set rule can never select again (memory only)
        for f in [f for f in com if w.sink_frames <= f < (i + 1) * w.chunk_frames - w.window_frames]:
            del com[f]
    fl = attn_flops(w.chunk_tokens, nk, w.head_dim, w.heads) * chunks
    per_layer_s = (t_append + t_attn) / chunks
    return {"value": fl / (t_append + t_attn) / 1e12, "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
            "sample": f"1 layer, {chunks} steady-state chunks, {w.heads} heads, {w.chunk_tokens} query rows x {nk} keys, "
                      f"fp64 numpy: attention {t_attn:.2f} s, append {t_append:.2f} s; "
                      f"x30 layers = {per_layer_s * 30:.0f} s per 30-layer chunk step (extrapolated)",
            "seconds": t_append + t_attn, "affinity_cores": len(os.sched_getaffinity(0)), "os_cpu_count": os.cpu_count()}


PEAK_FP8_TFLOPS = 2 * PEAK_BF16_TFLOPS      # dense fp8 MFMA peak (published: 5.0 PFLOP/s)


def copy_reference(nbytes, pool=10, reps=3):
    """Median time of a plain device-to-device copy of `nbytes` (read) + `nbytes` (written), each copy from and to
    buffers not touched since more than 256 MB of other traffic (HIP events around every copy, as around the appends)."""
    import torch
    src = [torch.full((nbytes,), i, dtype=torch.uint8, device="cuda") for i in range(pool)]
    dst = [torch.empty(nbytes, dtype=torch.uint8, device="cuda") for _ in range(pool)]
    t = []
    for rep in range(reps + 1):
        ev = []
        for i in range(pool):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            dst[i].copy_(src[i])
            b.record()
            ev.append((a, b))
        torch.cuda.synchronize()
        if rep:
            t += [a.elapsed_time(b) * 1e3 for a, b in ev]
    t.sort()
    med = t[len(t) // 2]
    return {"bytes_read": nbytes, "bytes_written": nbytes, "us_median": round(med, 2),
            "GBps": round(2 * nbytes / (med * 1e-6) / 1e9, 1), "copies": len(t)}


def single_layer_stats(w, gen, warmup=10, iters=50, kv_format="bf16", sink_relative=False):
    """Attention launch times of one layer in steady state: median, p10, p90 over `iters` launches (HIP events)."""
    import torch
    from paper_2509_22622_amd import binding
    Hh, D, Cf = w.heads, w.head_dim, w.chunk_frames
    nq = w.chunk_tokens
    nk = (w.sink_frames + w.window_frames + Cf) * w.tokens_per_frame
    cache = binding.Cache(1, Hh, D, w.grid_h, w.grid_w, Cf, w.sink_frames, w.window_frames, kv_format=kv_format)
    if sink_relative:
        cache.set_sink_relative(True)
    q, k, v = (torch.randn((nq, Hh, D), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16) for _ in range(3))
    qr, out = torch.empty(q.shape, dtype=torch.bfloat16 if kv_format == "bf16" else torch.uint8, device="cuda"), torch.empty_like(q)
    for c in range((w.sink_frames + w.window_frames) // Cf + 2):
        cache.chunk_append(0, c * Cf, Cf, q, k, v, qr)
    assert sum(b - a for a, b in cache.live_ranges(0)) == nk
    for _ in range(warmup):
        cache.sink_window_attn(0, qr, out)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
    for a, b in ev:
        a.record()
        cache.sink_window_attn(0, qr, out)
        b.record()
    torch.cuda.synchronize()
    ms = sorted(a.elapsed_time(b) for a, b in ev)
    med = ms[len(ms) // 2]
    fl = attn_flops(nq, nk, D, Hh)
    cache.close()
    res = {"workload": f"{w.name}: {nq} queries x {nk} keys x {Hh} heads x {D}", "launches": iters,
           "ms_median": round(med, 4), "ms_p10": round(ms[len(ms) // 10], 4), "ms_p90": round(ms[(len(ms) * 9) // 10], 4),
           "TFLOP/s": round(fl / (med * 1e-3) / 1e12, 1)}
    if kv_format == "bf16":
        res["pct_of_bf16_mfma_peak"] = round(100 * fl / (med * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 2)
    else:
        res["pct_of_fp8_mfma_peak"] = round(100 * fl / (med * 1e-3) / 1e12 / PEAK_FP8_TFLOPS, 2)
    return res


def prompt_side_stats(w, gen, n_text=512, reps=10):
    """The prompt side of KV-recache: cross-attention of one chunk's and of one re-prefill's queries over a prompt of
    `n_text` tokens, 30 layers back to back (HIP events around the 30 launches), and the replacement of the prompt's
    keys and values in all layers."""
    import torch
    from paper_2509_22622_amd import binding
    L, Hh, D = w.layers, w.heads, w.head_dim
    prompt = binding.Prompt(L, Hh, D, n_text)
    k, v = (torch.randn((n_text, Hh, D), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16) for _ in range(2))
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed(fn):
        for _ in range(3):
            fn()
        best = []
        for _ in range(reps):
            e0.record()
            fn()
            e1.record()
            torch.cuda.synchronize()
            best.append(e0.elapsed_time(e1))
        return sorted(best)[len(best) // 2]

    def switch():
        for l in range(L):
            prompt.recache(l, k, v)

    res = {"what": "cross-attention over the active prompt's keys (bf16, no mask, no rotary step) and the replacement "
                   "of those keys at a prompt switch; not part of `value`",
           "prompt_tokens": n_text,
           "switch_ms_30_layers": round(timed(switch), 4)}
    for name, nq in (("chunk", w.chunk_tokens), ("reprefill", 5 * w.chunk_tokens)):
        q = torch.randn((nq, Hh, D), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        out = torch.empty_like(q)

        def run():
            for l in range(L):
                prompt.cross_attn(l, q, out)

        ms = timed(run)
        fl = attn_flops(nq, n_text, D, Hh) * L
        by = (2 * nq + 2 * n_text) * Hh * D * 2 * L
        res[name] = {"queries": nq, "ms_30_layers": round(ms, 4), "us_per_layer": round(ms * 1e3 / L, 2),
                     "TFLOP/s": round(fl / (ms * 1e-3) / 1e12, 1),
                     "pct_of_bf16_mfma_peak": round(100 * fl / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 2),
                     "algorithmic_GBps": round(by / (ms * 1e-3) / 1e9, 1)}
        # the block's whole output path: attention, then y = concat_heads(out) w^T with one weight per layer
        n = Hh * D
        if name == "chunk":
            w_row = (torch.randn((L, n, n), generator=gen, device="cuda", dtype=torch.float32) / n ** 0.5).to(torch.bfloat16)
            w_out = torch.empty_like(w_row)                  # packed once, as at model load
            for l in range(L):
                prompt.pack_out_weight(w_row[l], w_out[l])
            del w_row
        y = torch.empty((nq, n), dtype=torch.bfloat16, device="cuda")
        work = torch.empty(prompt.cross_attn_out_workspace_bytes(nq), dtype=torch.uint8, device="cuda")

        def run_out():
            for l in range(L):
                prompt.cross_attn_out(l, q, w_out[l], work, y)

        ms_out = timed(run_out)
        fl_proj = 2.0 * nq * n * n * L
        res[name]["with_out_projection"] = {
            "ms_30_layers": round(ms_out, 4), "us_per_layer": round(ms_out * 1e3 / L, 2),
            "projection_us_per_layer": round((ms_out - ms) * 1e3 / L, 2),
            "projection_TFLOP/s": round(fl_proj / ((ms_out - ms) * 1e-3) / 1e12, 1),
            "projection_pct_of_bf16_mfma_peak": round(100 * fl_proj / ((ms_out - ms) * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 2),
            "block_TFLOP/s": round((fl + fl_proj) / (ms_out * 1e-3) / 1e12, 1)}
    prompt.close()
    return res


def train_step_stats(w, gen, clip_frames=21, reps=5):
    """The train-time rule at the benchmark model's layer shape: forward of a supervised clip of `clip_frames` frames
    over sink + a full detached window + itself, and the backward pass (HIP events; one layer)."""
    import torch
    from paper_2509_22622_amd import binding
    Hh, D, C, S, W, T = w.heads, w.head_dim, w.chunk_frames, w.sink_frames, w.window_frames, clip_frames
    P = w.tokens_per_frame
    clip = binding.Clip(Hh, D, w.grid_h, w.grid_w, C, S, W, T)
    rnd = lambda n: torch.randn((n * P, Hh, D), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    q, k, v, dout = rnd(T), rnd(S + W + T), rnd(S + W + T), rnd(T)
    out, dq, dk, dv = (torch.empty_like(q) for _ in range(4))
    ev = lambda: torch.cuda.Event(enable_timing=True)
    tf, tb = [], []
    for _ in range(reps + 1):
        a, b, c = ev(), ev(), ev()
        a.record()
        clip.forward(60, W, T, q, k, v, out)
        b.record()
        clip.backward(dout, dq, dk, dv)
        c.record()
        torch.cuda.synchronize()
        tf.append(a.elapsed_time(b))
        tb.append(b.elapsed_time(c))
    tf, tb = sorted(tf[1:])[reps // 2], sorted(tb[1:])[reps // 2]
    pairs = ((T + C - 1) // C) * (C * P) * ((S + W + C) * P)          # every chunk sees sink + W frames + itself
    # pairs whose key belongs to the clip (only those keys receive dK and dV): a clip frame is seen by its own chunk
    # and by the later chunks that start within W frames after it
    n_chunks = (T + C - 1) // C
    clip_pairs = sum((min(n_chunks - 1, (g + W) // C) - g // C + 1) * C * P * P for g in range(T))
    fl = attn_flops(1, 1, D, Hh) * pairs
    one = fl / 2                                                      # one product over all unmasked pairs
    fl_bwd = 3 * one + 2 * one * clip_pairs / pairs                   # scores' dP, dQ over all pairs; dK, dV over the clip's keys
    fl_bwd_run = 3 * one + 4 * one * clip_pairs / pairs               # what the two kernels execute (scores and dP in both)
    res = {"what": "attention of a supervised clip over sink + detached window + itself and its gradients (bf16; one "
                   "layer); not part of `value`",
           "workload": f"{w.name}-shaped clip: {T} frames in chunks of {C}, sink {S}, window {W}: {T * P} queries, "
                       f"{(S + W + T) * P} resident keys, {Hh} heads x {D}",
           "workspace_bytes": int(clip.buffer.numel()),
           "forward_ms": round(tf, 3), "forward_TFLOP/s": round(fl / (tf * 1e-3) / 1e12, 1),
           "backward_ms": round(tb, 3),
           "backward_TFLOP/s": round(fl_bwd / (tb * 1e-3) / 1e12, 1),
           "backward_pct_of_bf16_mfma_peak": round(100 * fl_bwd / (tb * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 2),
           "backward_executed_TFLOP/s": round(fl_bwd_run / (tb * 1e-3) / 1e12, 1),
           "flops": "forward: 2 products (4 Nq Nk D H) over the unmasked pairs; backward: dP, dQ and the scores again "
                    "over all pairs, dK and dV over the pairs whose key is a clip frame (context and sink keys get no "
                    f"gradient: {clip_pairs / pairs:.3f} of the pairs); executed: scores and dP in both kernels",
           "forward_TFLOP": round(fl / 1e12, 3), "backward_TFLOP": round(fl_bwd / 1e12, 3),
           "backward_executed_TFLOP": round(fl_bwd_run / 1e12, 3)}
    clip.close()
    return res


def fp8_cache_stats(w_loop, gen, q, k, v, steps, only_step=False, variant=0):
    """The 8-bit (E4M3) cache variant: a different accuracy tier, reported next to the bf16 figures and never as
    `value`.  Single-layer launch statistics, the 30-layer chunk step (append + attention, wall clock), and the
    distance between the two paths' outputs on the same inputs."""
    import torch
    from paper_2509_22622_amd import binding, synth
    w = w_loop
    L, Hh, D, Cf = w.layers, w.heads, w.head_dim, w.chunk_frames
    nq = w.chunk_tokens
    nk = (w.sink_frames + w.window_frames + Cf) * w.tokens_per_frame
    res = {"what": "K', V and q' held as 8-bit floating point (OCP E4M3), both products on the fp8 MFMA: reduced "
                   "precision, not the benchmark's metric"}
    if not only_step:
        res["single_layer"] = {"cfg2": single_layer_stats(synth.WAN_LAYER, gen, kv_format="fp8_e4m3"),
                               "cfg4": single_layer_stats(synth.LONG_WINDOW, gen, kv_format="fp8_e4m3")}
        names = {n: i for i, n in binding.attn_variant_names().items()}
        if "d128_fp8_loglin" in names:      # the cheaper weights (a linear map to the E4M3 code instead of exp2)
            binding.set_attn_variant(names["d128_fp8_loglin"])
            try:
                res["single_layer"]["cfg2_loglin_weights"] = single_layer_stats(synth.WAN_LAYER, gen, kv_format="fp8_e4m3")
            finally:
                binding.set_attn_variant(variant)
        res.update(_fp8_vs_bf16(q, k, v, L, Hh, D, Cf))
    return _fp8_step(res, w, q, k, v, steps)


def _fp8_vs_bf16(q, k, v, L, Hh, D, Cf):
    """Distance between the two paths' outputs: one layer, six chunks streamed into both kinds of cache."""
    import torch
    from paper_2509_22622_amd import binding, synth
    res = {}
    wl = synth.WAN_LAYER
    ca = binding.Cache(1, Hh, D, wl.grid_h, wl.grid_w, Cf, wl.sink_frames, wl.window_frames)
    cb = binding.Cache(1, Hh, D, wl.grid_h, wl.grid_w, Cf, wl.sink_frames, wl.window_frames, kv_format="fp8_e4m3")
    qa, oa = torch.empty_like(q[0, 0]), torch.empty_like(q[0, 0])
    qb, ob = torch.empty(q[0, 0].shape, dtype=torch.uint8, device="cuda"), torch.empty_like(q[0, 0])
    for c in range(6):
        i, l = c % q.shape[0], c % L
        ca.chunk_append(0, c * Cf, Cf, q[i, l], k[i, l], v[i, l], qa)
        cb.chunk_append(0, c * Cf, Cf, q[i, l], k[i, l], v[i, l], qb)
    ca.sink_window_attn(0, qa, oa)
    cb.sink_window_attn(0, qb, ob)
    torch.cuda.synchronize()
    d = (ob.float() - oa.float())
    res["rel_l2_vs_bf16_path"] = round(float(d.norm() / oa.float().norm()), 5)
    res["max_abs_vs_bf16_path"] = round(float(d.abs().max()), 5)
    ca.close()
    cb.close()
    return res


def _fp8_step(res, w, q, k, v, steps):
    """The 30-layer chunk step (append + attention per layer) over the 8-bit cache, wall clock."""
    import torch
    from paper_2509_22622_amd import binding
    L, Hh, D, Cf = w.layers, w.heads, w.head_dim, w.chunk_frames
    nq = w.chunk_tokens
    nk = (w.sink_frames + w.window_frames + Cf) * w.tokens_per_frame
    cache = binding.Cache(L, Hh, D, w.grid_h, w.grid_w, Cf, w.sink_frames, w.window_frames, kv_format="fp8_e4m3")
    res["cache_bytes"] = int(cache.buffer.numel())
    qr = torch.empty((L, nq, Hh, D), dtype=torch.uint8, device="cuda")
    out = torch.empty((L, nq, Hh, D), dtype=torch.bfloat16, device="cuda")
    chunk = 0
    pool = q.shape[0]

    def step(attn=True):
        nonlocal chunk
        f0, i = chunk * Cf, chunk % pool
        for l in range(L):
            cache.chunk_append(l, f0, Cf, q[i, l], k[i, l], v[i, l], qr[l])
            if attn:
                cache.sink_window_attn(l, qr[l], out[l])
        chunk += 1

    for _ in range((w.sink_frames + w.window_frames) // Cf + 1):
        step(attn=False)
    for _ in range(2):
        step()
    assert sum(b - a for a, b in cache.live_ranges(0)) == nk
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / steps * 1e3
    fl = attn_flops(nq, nk, D, Hh) * L
    res["step_30_layers"] = {"ms_per_step": round(ms, 4), "TFLOP/s": round(fl / (ms * 1e-3) / 1e12, 1),
                             "pct_of_fp8_mfma_peak": round(100 * fl / (ms * 1e-3) / 1e12 / PEAK_FP8_TFLOPS, 2), "steps": steps}
    if "single_layer" in res:
        # the recache workload (sink 3 + 12 window frames at a late position, chunk-causal), 30 layers
        from paper_2509_22622_amd import synth
        wr = synth.RECACHE
        nf = wr.sink_frames + wr.window_frames + wr.chunk_frames
        rshape = (nf * w.tokens_per_frame, Hh, D)
        gen = torch.Generator(device="cuda")
        gen.manual_seed(synth.MASTER_SEED + 5)
        rq, rk, rv = (torch.randn(rshape, generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16) for _ in range(3))
        ro = torch.empty(rshape, dtype=torch.bfloat16, device="cuda")
        ws = chunk * Cf - (wr.window_frames + wr.chunk_frames)

        def recache():
            for l in range(L):
                cache.recache_prefill(l, True, ws, wr.window_frames + wr.chunk_frames, rq, rk, rv, ro)

        recache()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(3):
            recache()
        torch.cuda.synchronize()
        r_ms = (time.perf_counter() - t0) / 3 * 1e3
        n_ch = nf // Cf
        pairs = sum(min(i + 1, (wr.sink_frames + wr.window_frames) // Cf + 1) for i in range(n_ch))
        r_fl = attn_flops(nq, nq, D, Hh) * pairs * L
        res["recache_prefill"] = {"ms_30_layers": round(r_ms, 3), "TFLOP/s": round(r_fl / (r_ms * 1e-3) / 1e12, 1)}
    cache.close()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--variant", type=int, default=0, help="attention kernel variant (0 = default)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--two-call-step", action="store_true",
                    help="time ll_chunk_append(q, q_out) + ll_sink_window_attn(q_out) instead of the pair that keeps the "
                         "rotated queries out of memory")
    ap.add_argument("--no-recache", action="store_true")
    ap.add_argument("--no-fp8", action="store_true", help="leave out the figures of the 8-bit cache variant")
    ap.add_argument("--fp8-only", action="store_true",
                    help="only the 30-layer step over the 8-bit cache (for profiler runs: one launch shape)")
    ap.add_argument("--prompt-only", action="store_true",
                    help="only the prompt side (cross-attention over the prompt, prompt switch), for profiler runs")
    ap.add_argument("--clip-only", action="store_true",
                    help="only the train-time rule (clip forward and backward), for profiler runs")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the graph replay, the single-layer statistics and the MFMA probe (for profiler runs)")
    ap.add_argument("--full-loop", action="store_true",
                    help="also run 60 consecutive chunks from an empty cache (30 layers), with a time per chunk")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (--gpus 1); heads are independent, so the path would shard by head")

    import torch
    from paper_2509_22622_amd import binding, synth
    if not os.path.exists(binding.LIB_PATH):
        from paper_2509_22622_amd import build as _b
        _b.build()
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    binding.set_attn_variant(args.variant)
    w = synth.WAN_LOOP
    L, Hh, D, P, Cf = w.layers, w.heads, w.head_dim, w.tokens_per_frame, w.chunk_frames
    nq = w.chunk_tokens
    nk = (w.sink_frames + w.window_frames + Cf) * P
    cache = binding.Cache(L, Hh, D, w.grid_h, w.grid_w, Cf, w.sink_frames, w.window_frames)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(synth.MASTER_SEED)
    pool = 2
    shape = (pool, L, nq, Hh, D)
    # generate layer by layer to keep the fp32 staging small
    def gen_bf16():
        t = torch.empty(shape, dtype=torch.bfloat16, device="cuda")
        for i in range(pool):
            for l in range(L):
                t[i, l] = torch.randn((nq, Hh, D), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        return t
    if args.clip_only:
        print(json.dumps({"train_step": train_step_stats(w, gen)}))
        return
    if args.prompt_only:
        print(json.dumps({"prompt_side": prompt_side_stats(w, gen)}))
        return
    q, k, v = gen_bf16(), gen_bf16(), gen_bf16()
    if args.fp8_only:
        print(json.dumps({"fp8_cache": fp8_cache_stats(w, gen, q, k, v, args.steps, only_step=True, variant=args.variant)}))
        return
    qr = torch.empty((L, nq, Hh, D), dtype=torch.bfloat16, device="cuda")
    out = torch.empty((L, nq, Hh, D), dtype=torch.bfloat16, device="cuda")

    chunk = 0
    def step(events=None):
        # HIP events cost a few microseconds each on the GPU's queue: only every tenth layer is bracketed
        nonlocal chunk
        f0, i = chunk * Cf, chunk % pool
        for l in range(L):
            timed = events is not None and l % 10 == 0
            if timed:
                e0, e1, e2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
                e0.record()
            if args.two_call_step:                 # rotated queries written by the append, read by the attention
                cache.chunk_append(l, f0, Cf, q[i, l], k[i, l], v[i, l], qr[l])
            else:                                  # keys and values only; the attention kernel turns the queries
                cache.chunk_append(l, f0, Cf, None, k[i, l], v[i, l], None)
            if timed:
                e1.record()
            if args.two_call_step:
                cache.sink_window_attn(l, qr[l], out[l])
            else:
                cache.sink_window_attn_unrotated(l, q[i, l], out[l])
            if timed:
                e2.record()
                events.append((e0, e1, e2))
        chunk += 1

    n_fill = (w.sink_frames + w.window_frames) // Cf + 1      # chunks until every ring slot is live
    for _ in range(n_fill):                                    # fill the caches: appends only, so that every
        f0, i = chunk * Cf, chunk % pool                       # attention launch of this run has the steady shape
        for l in range(L):
            if args.two_call_step:
                cache.chunk_append(l, f0, Cf, q[i, l], k[i, l], v[i, l], qr[l])
            else:
                cache.chunk_append(l, f0, Cf, None, k[i, l], v[i, l], None)
        chunk += 1
    for _ in range(args.warmup):
        step()
    assert sum(b - a for a, b in cache.live_ranges(0)) == nk
    torch.cuda.synchronize()
    events = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(events)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    append_ms = sum(a.elapsed_time(b) for a, b, _ in events) / len(events)
    attn_ms = sum(b.elapsed_time(c) for _, b, c in events) / len(events)
    fl_layer = attn_flops(nq, nk, D, Hh)
    tflops = fl_layer * L / (ms_per_step * 1e-3) / 1e12
    attn_tflops = fl_layer / (attn_ms * 1e-3) / 1e12
    # read q, k, v + write q', K', V; without the queries when the attention kernel turns them itself
    append_bytes = (6 if args.two_call_step else 4) * nq * Hh * D * 2
    res = {
        "metric": "sink+window attn TFLOP/s & ms per 3-frame chunk (30 layers); % bf16 MFMA peak",
        "value": round(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "wan1.3b-30layers: 30 layers x (12 heads x 128, 1560 tok/frame, chunk 3, sink 3, window 9; "
                               "4680 queries x 23400 keys), steady state, append + attention per layer"
                               + ("" if args.two_call_step else " (ll_chunk_append of keys and values, ll_sink_window_attn_unrotated)"),
                   "attn_variant": binding.attn_variant_names().get(args.variant, "default")},
        "pct_of_bf16_mfma_peak": round(100 * tflops / PEAK_BF16_TFLOPS, 2),
        "attn_ms_per_layer": round(attn_ms, 4), "append_ms_per_layer": round(append_ms, 4),
        "append_GBps": round(append_bytes / (append_ms * 1e-3) / 1e9, 1),
        "roofline": {"bound": "mfma", "kernel": "ll_attn_stream16_kernel<128, false, false, %d>" % (9 if args.two_call_step else 25), "achieved": round(attn_tflops, 2), "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(attn_tflops / PEAK_BF16_TFLOPS, 4), "traffic": ATTN_HBM_TRAFFIC_BYTES,
                     "traffic_source": ATTN_HBM_TRAFFIC_SOURCE,
                     "flops_per_launch": fl_layer, "avg_launch_ms": round(attn_ms, 4),
                     "algorithmic_bytes": (2 * nq + 2 * nk) * Hh * D * 2},
    }

    # What a plain device copy of the append's bytes achieves from buffers that are in no cache: the practical bound
    # of the memory-bound append (and, under rocprofv3 --pmc, the dispatch of known size that scales the counters).
    res["append_copy_reference"] = copy_reference(append_bytes // 2)
    res["append_vs_copy_reference"] = round(res["append_copy_reference"]["us_median"] / (append_ms * 1e3), 3)

    if args.no_extras:
        print(json.dumps(res))
        return

    # The other form of the same step, for comparison: the one not timed above.
    def other_step():
        nonlocal chunk
        f0, i = chunk * Cf, chunk % pool
        for l in range(L):
            if args.two_call_step:
                cache.chunk_append(l, f0, Cf, None, k[i, l], v[i, l], None)
                cache.sink_window_attn_unrotated(l, q[i, l], out[l])
            else:
                cache.chunk_append(l, f0, Cf, q[i, l], k[i, l], v[i, l], qr[l])
                cache.sink_window_attn(l, qr[l], out[l])
        chunk += 1
    other_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        other_step()
    torch.cuda.synchronize()
    o_ms = (time.perf_counter() - t0) / args.steps * 1e3
    res["other_form_of_the_step"] = {
        "ms_per_step": round(o_ms, 4), "TFLOP/s": round(fl_layer * L / (o_ms * 1e-3) / 1e12, 2),
        "what": ("keys and values appended, queries turned by the attention kernel" if args.two_call_step else
                 "ll_chunk_append(q, q_out) + ll_sink_window_attn(q_out): the rotated queries go through memory")}

    # The repeated denoising passes of one chunk (same frames, new contents) as one captured HIP graph: the
    # 60 launches of a step replayed without per-launch host work.
    f0g, ig = (chunk - 1) * Cf, (chunk - 1) % pool
    def repass():
        for l in range(L):
            if args.two_call_step:
                cache.chunk_append(l, f0g, Cf, q[ig, l], k[ig, l], v[ig, l], qr[l])
                cache.sink_window_attn(l, qr[l], out[l])
            else:
                cache.chunk_append(l, f0g, Cf, None, k[ig, l], v[ig, l], None)
                cache.sink_window_attn_unrotated(l, q[ig, l], out[l])
    repass()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        repass()
    graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        graph.replay()
    torch.cuda.synchronize()
    g_ms = (time.perf_counter() - t0) / args.steps * 1e3
    res["graph_replay"] = {"ms_per_step": round(g_ms, 4), "TFLOP/s": round(fl_layer * L / (g_ms * 1e-3) / 1e12, 2),
                           "what": "one captured graph = 30 x (append of the staged chunk again, attention); a denoising re-pass"}

    if not args.no_recache:
        # KV-recache prefill, config 5: sink 3 + 12 window frames at a late position, per layer, 30 layers
        wr = synth.RECACHE
        nf = wr.sink_frames + wr.window_frames + wr.chunk_frames
        rshape = (nf * P, Hh, D)
        rq, rk, rv = (torch.randn(rshape, generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16) for _ in range(3))
        ro = torch.empty(rshape, dtype=torch.bfloat16, device="cuda")
        ws = chunk * Cf - (wr.window_frames + wr.chunk_frames)
        def recache():
            for l in range(L):
                cache.recache_prefill(l, True, ws, wr.window_frames + wr.chunk_frames, rq, rk, rv, ro)
        recache()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        reps = 3
        for _ in range(reps):
            recache()
        torch.cuda.synchronize()
        r_ms = (time.perf_counter() - t0) / reps * 1e3
        n_ch = nf // Cf
        pairs = sum(min(i + 1, (wr.sink_frames + wr.window_frames) // Cf + 1) for i in range(n_ch))
        r_fl = attn_flops(nq, nq, D, Hh) * pairs * L
        res["recache_prefill"] = {"ms_30_layers": round(r_ms, 3), "TFLOP/s": round(r_fl / (r_ms * 1e-3) / 1e12, 2),
                                  "workload": f"{nf} frames = {n_ch} chunks, chunk-causal, {nf * P} queries, 30 layers"}

    if args.full_loop:
        # config 3 as a whole: warm-up chunks included, the ring of 4 chunk slots wraps 14 times
        for l in range(L):
            cache.reset(l)
        torch.cuda.synchronize()
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(61)]
        marks[0].record()
        for c in range(60):
            i = c % pool
            for l in range(L):
                if args.two_call_step:
                    cache.chunk_append(l, c * Cf, Cf, q[i, l], k[i, l], v[i, l], qr[l])
                    cache.sink_window_attn(l, qr[l], out[l])
                else:
                    cache.chunk_append(l, c * Cf, Cf, None, k[i, l], v[i, l], None)
                    cache.sink_window_attn_unrotated(l, q[i, l], out[l])
            marks[c + 1].record()
        torch.cuda.synchronize()
        per_chunk = [marks[c].elapsed_time(marks[c + 1]) for c in range(60)]
        steady = sorted(per_chunk[4:])
        res["full_loop"] = {"ms_per_chunk": [round(x, 3) for x in per_chunk], "median_ms_chunks_4_to_59": round(steady[len(steady) // 2], 3),
                            "total_ms": round(sum(per_chunk), 2)}

    # single-layer launches back to back (no appends in between): the Wan layer and the long window it replaces
    import dataclasses
    wan14b = dataclasses.replace(synth.WAN_LAYER, name="wan14b-shaped-layer", heads=40)      # 40 heads: three rounds of tiles
    res["single_layer"] = {"cfg2": single_layer_stats(synth.WAN_LAYER, gen), "cfg4": single_layer_stats(synth.LONG_WINDOW, gen),
                           "heads40": single_layer_stats(wan14b, gen, warmup=5, iters=20),
                           # the sink at a fixed rotary distance from the window (its own range, queries turned for it)
                           "cfg2_sink_relative": single_layer_stats(synth.WAN_LAYER, gen, sink_relative=True)}

    # What a pure MFMA stream sustains on this GPU right now (diagnostic kernel of the library): the chip is
    # power-limited under a full matrix load, far below the boost clock when the operand bits toggle.
    pr_t, pr_c = binding.probe_mfma_rate(256, 20000, True)
    pc_t, pc_c = binding.probe_mfma_rate(256, 20000, False)
    res["mfma_probe"] = {"random_operands": {"TFLOP/s": round(pr_t, 1), "clock_GHz": round(pr_c, 3)},
                         "constant_operands": {"TFLOP/s": round(pc_t, 1), "clock_GHz": round(pc_c, 3)},
                         "workload": "256 workgroups x 8 waves, 32x32x16 bf16 MFMAs back to back",
                         "attn_kernel_vs_random_operand_probe": round(attn_tflops / pr_t, 4)}

    res["prompt_side"] = prompt_side_stats(w, gen)
    res["train_step"] = train_step_stats(w, gen)

    if not args.no_fp8:
        res["fp8_cache"] = fp8_cache_stats(w, gen, q, k, v, args.steps, variant=args.variant)

    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(synth.WAN_LAYER)
    print(json.dumps(res))


if __name__ == "__main__":
    main()

"""The calls enqueue work and touch no allocator, so a caller can capture them in a HIP graph.  A replay re-runs the
staged chunk's append and attention on whatever the captured tensors hold now: the repeated denoising passes of one
chunk (Alg. 2), with the launch overhead of the 2 x layers kernels paid once."""
import numpy as np
import pytest
import torch

from paper_2509_22622_amd import binding as B
from paper_2509_22622_amd import synth
from oracle.fp8_cache import Fp8Oracle
from oracle.longlive_oracle import Oracle

import gpu_harness as H
from test_gpu_fp8 import assert_parity8

pytestmark = pytest.mark.gpu

W = synth.Workload("graph-mid", 91, 3, 4, 128, 6, 10, 3, 3, 6, 8)


@pytest.mark.parametrize("kv_format", ["bf16", "fp8_e4m3"])
def test_graph_replay_equals_eager_passes(kv_format):
    P, C = W.tokens_per_frame, W.chunk_frames
    fp8 = kv_format != "bf16"
    make = (lambda: B.Cache(W.layers, W.heads, W.head_dim, W.grid_h, W.grid_w, C, W.sink_frames, W.window_frames,
                            kv_format=kv_format))
    eager, graphed = make(), make()
    oracle = Fp8Oracle(H.oracle_cfg(W)) if fp8 else Oracle(H.oracle_cfg(W))
    qdt = torch.uint8 if fp8 else torch.bfloat16            # rotated queries: E4M3 bytes in the 8-bit variant
    shape = (C * P, W.heads, W.head_dim)
    hist = 5
    for i in range(hist):                                   # same history in both caches (and the oracle, layer 0)
        for l in range(W.layers):
            q, k, v = synth.chunk_qkv(W, l, i)
            qd, kd, vd = H.to_dev(q), H.to_dev(k), H.to_dev(v)
            for c in (eager, graphed):
                c.chunk_append(l, i * C, C, qd, kd, vd, torch.empty(qd.shape, dtype=qdt, device="cuda"))
            if l == 0:
                oracle.append(0, i * C, q, k, v)
    f0 = hist * C
    sq, sk, sv = (torch.zeros((W.layers,) + shape, dtype=torch.bfloat16, device="cuda") for _ in range(3))
    sqr, sout = torch.empty(sq.shape, dtype=qdt, device="cuda"), torch.empty_like(sq)

    def one_pass(cache, q, k, v, qr, out):
        for l in range(W.layers):
            cache.chunk_append(l, f0, C, q[l], k[l], v[l], qr[l])
            cache.sink_window_attn(l, qr[l], out[l])

    one_pass(graphed, sq, sk, sv, sqr, sout)                # eager once: kernels loaded, attributes set, chunk staged
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        one_pass(graphed, sq, sk, sv, sqr, sout)
    for rep in range(4):                                    # four denoising passes with fresh contents
        host = [synth.chunk_qkv(W, l, 100 + rep) for l in range(W.layers)]
        q, k, v = (torch.stack([H.to_dev(h[t]) for h in host]) for t in range(3))
        qr, out = torch.empty(q.shape, dtype=qdt, device="cuda"), torch.empty_like(q)
        one_pass(eager, q, k, v, qr, out)                   # the program's own eager work between replays
        torch.cuda.synchronize()
        sq.copy_(q), sk.copy_(k), sv.copy_(v)
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(sout.view(torch.int16), out.view(torch.int16)), f"replay {rep}"
        assert torch.equal(sqr, qr), f"replay {rep}"
        assert graphed.live_frames(0) == eager.live_frames(0)
        oracle.append(0, f0, *host[0])                      # same f0: overwrites the staged chunk
        if fp8:
            vmax = max(np.abs(oracle.frame_kv(0, f)[1]).max() for f in oracle.live_frames(0))
            assert_parity8(H.to_bits(sout[0]), oracle.attn(0), vmax, f"replay {rep} vs oracle")
        else:
            H.assert_parity(H.to_bits(sout[0]), oracle.attn(0), f"replay {rep} vs oracle")
    # the next chunk commits the staged one in both caches alike
    q, k, v = synth.chunk_qkv(W, 0, 200)
    qd, kd, vd = H.to_dev(q), H.to_dev(k), H.to_dev(v)
    outs = []
    for c in (eager, graphed):
        qr, o = torch.empty(qd.shape, dtype=qdt, device="cuda"), torch.empty_like(qd)
        c.chunk_append(0, f0 + C, C, qd, kd, vd, qr)
        c.sink_window_attn(0, qr, o)
        outs.append(o)
    torch.cuda.synchronize()
    assert torch.equal(outs[0].view(torch.int16), outs[1].view(torch.int16))
    eager.close()
    graphed.close()


def test_graph_replay_of_the_unrotated_query_pair():
    """ll_chunk_append(keys and values only) + ll_sink_window_attn_unrotated captured in a HIP graph: the cache write
    leaves the frame-axis table for the attention kernel with a plain store (no memset node, no host copy), so replays
    with fresh contents match the eager two-call path bit for bit, and the oracle."""
    P, C = W.tokens_per_frame, W.chunk_frames
    make = lambda: B.Cache(W.layers, W.heads, W.head_dim, W.grid_h, W.grid_w, C, W.sink_frames, W.window_frames)
    eager, graphed, oracle = make(), make(), Oracle(H.oracle_cfg(W))
    shape = (C * P, W.heads, W.head_dim)
    hist = 5
    for i in range(hist):
        for l in range(W.layers):
            q, k, v = synth.chunk_qkv(W, l, i)
            qd, kd, vd = H.to_dev(q), H.to_dev(k), H.to_dev(v)
            eager.chunk_append(l, i * C, C, qd, kd, vd, torch.empty_like(qd))
            graphed.chunk_append(l, i * C, C, None, kd, vd, None)
            if l == 0:
                oracle.append(0, i * C, q, k, v)
    f0 = hist * C
    sq, sk, sv = (torch.zeros((W.layers,) + shape, dtype=torch.bfloat16, device="cuda") for _ in range(3))
    sout = torch.empty_like(sq)

    def fused_pass():
        for l in range(W.layers):
            graphed.chunk_append(l, f0, C, None, sk[l], sv[l], None)
            graphed.sink_window_attn_unrotated(l, sq[l], sout[l])

    fused_pass()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        fused_pass()
    for rep in range(4):
        host = [synth.chunk_qkv(W, l, 300 + rep) for l in range(W.layers)]
        q, k, v = (torch.stack([H.to_dev(h[t]) for h in host]) for t in range(3))
        qr, out = torch.empty_like(q), torch.empty_like(q)
        for l in range(W.layers):                           # the program's own eager work between replays
            eager.chunk_append(l, f0, C, q[l], k[l], v[l], qr[l])
            eager.sink_window_attn(l, qr[l], out[l])
        torch.cuda.synchronize()
        sq.copy_(q), sk.copy_(k), sv.copy_(v)
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(sout.view(torch.int16), out.view(torch.int16)), f"replay {rep}"
        oracle.append(0, f0, *host[0])
        H.assert_parity(H.to_bits(sout[0]), oracle.attn(0), f"replay {rep} vs oracle")
    eager.close()
    graphed.close()

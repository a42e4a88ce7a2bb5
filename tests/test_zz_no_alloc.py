"""ll_recache_prefill_static (the re-prefill for callers that cannot allocate or hand over scratch memory: the E4M3
queries of an 8-bit cache are staged in an array inside the library) against ll_recache_prefill, through the C-ABI.

Both calls run the same kernels on the same inputs, so outputs, cache contents and bookkeeping must agree bit for
bit.  Two calls in a row on one GPU, the second with a smaller input (the array keeps the first call's queries),
then the size limit's error and a bf16 handle, for which the call is the plain re-prefill.
"""
import numpy as np
import pytest
import torch

from paper_2509_22622_amd import binding as B
from paper_2509_22622_amd import synth

import gpu_harness as H

pytestmark = pytest.mark.gpu

W1 = synth.Workload("noalloc-a", 901, 2, 3, 128, 9, 15, 3, 3, 6, 8)      # P = 135: ragged tiles; two layers
W2 = synth.Workload("noalloc-b", 902, 1, 2, 64, 5, 7, 3, 2, 5, 8)        # smaller, D = 64, S % C != 0


def _cache8(w):
    return B.Cache(w.layers, w.heads, w.head_dim, w.grid_h, w.grid_w, w.chunk_frames, w.sink_frames, w.window_frames,
                   kv_format="fp8_e4m3")


def _history(cache, w, layer, n_chunks):
    for i in range(n_chunks):
        q, k, v = (H.to_dev(t) for t in synth.chunk_qkv(w, layer, i))
        cache.chunk_append(layer, i * w.chunk_frames, w.chunk_frames, q, k, v,
                           torch.empty(q.shape, dtype=torch.uint8, device="cuda"))


def _frames(cache, w, layer):
    out = []
    for f in cache.live_frames(layer):
        kd = torch.empty((w.tokens_per_frame, w.heads, w.head_dim), dtype=torch.uint8, device="cuda")
        vd = torch.empty_like(kd)
        cache.read_frame(layer, f, kd, vd)
        out += [kd, vd]
    torch.cuda.synchronize()
    return out


def _both(w, layer, include_sink, ws, n_win, seed):
    """The same re-prefill through both entry points on two caches with the same history; returns the output."""
    a, b = _cache8(w), _cache8(w)
    _history(a, w, layer, 5)
    _history(b, w, layer, 5)
    nf = (w.sink_frames if include_sink else 0) + n_win
    shape = (nf * w.tokens_per_frame, w.heads, w.head_dim)
    q, k, v = (H.to_dev(synth.normal_bf16(shape, w.cfg_id, layer, seed, t)) for t in "qkv")
    out_a = torch.full(shape, 7.0, dtype=torch.bfloat16, device="cuda")
    out_b = torch.full(shape, -7.0, dtype=torch.bfloat16, device="cuda")
    a.recache_prefill(layer, include_sink, ws, n_win, q, k, v, out_a)
    b.recache_prefill_static(layer, include_sink, ws, n_win, q, k, v, out_b)
    torch.cuda.synchronize()
    assert torch.isfinite(out_a.float()).all()
    assert torch.equal(out_a.view(torch.int16), out_b.view(torch.int16)), f"{w.name}: outputs differ"
    assert a.live_frames(layer) == b.live_frames(layer)
    for x, y in zip(_frames(a, w, layer), _frames(b, w, layer)):
        assert torch.equal(x, y), f"{w.name}: cache contents differ"
    # the two caller-owned buffers differ in exactly one place: the plain call staged its E4M3 queries in its buffer,
    # the static call left that area as ll_cache_create zeroed it (its queries went to the library's own array)
    differ = a.buffer != b.buffer
    assert int(differ.sum()) > shape[0] * shape[1] * shape[2] // 2          # most codes of N(0,1) queries are not 0
    assert bool((b.buffer[differ] == 0).all())
    # streaming goes on from both caches alike
    f0 = ws + n_win
    q, k, v = (H.to_dev(t) for t in synth.chunk_qkv(w, layer, 77))
    res = []
    for c in (a, b):
        qr = torch.empty(q.shape, dtype=torch.uint8, device="cuda")
        o = torch.empty_like(q)
        c.chunk_append(layer, f0, w.chunk_frames, q, k, v, qr)
        c.sink_window_attn(layer, qr, o)
        res.append(o)
    torch.cuda.synchronize()
    assert torch.equal(res[0].view(torch.int16), res[1].view(torch.int16))
    a.close()
    b.close()
    return out_b


def test_static_staging_equals_the_cache_buffers_staging():
    big = _both(W1, 1, True, 40, 9, 1)            # 12 frames x 135 tokens x 3 heads x 128
    small = _both(W2, 0, False, 21, 7, 2)         # right after it, smaller: 7 frames x 35 tokens x 2 heads x 64
    assert big.numel() > 4 * small.numel()
    again = _both(W1, 0, True, 9, 4, 3)           # and a third, between the two in size, sink + a short window
    assert again.shape[0] == 7 * W1.tokens_per_frame


def test_size_limit_and_bf16_handle():
    L = B.lib()
    # 36 MiB hold 15 frames of 1560 tokens x 12 heads x 128 (34.3 MiB), not 15 frames of 1560 x 14 x 128
    w = synth.Workload("too-big", 903, 1, 14, 128, 30, 52, 3, 3, 9, 1)
    c = _cache8(w)
    shape = (15 * w.tokens_per_frame, w.heads, w.head_dim)
    q = torch.zeros(shape, dtype=torch.bfloat16, device="cuda")
    out = torch.empty_like(q)
    with pytest.raises(B.LongLiveError) as e:
        c.recache_prefill_static(0, True, 30, 12, q, q, q, out)
    assert e.value.status == B.LL_ERR_BUFFER_TOO_SMALL and "static area" in str(e.value)
    assert c.live_frames(0) == []                                    # nothing was enqueued, nothing changed
    c.close()
    # a bf16 cache needs no scratch: the call is the plain re-prefill, bit for bit
    wb = W2
    a, b = H.make_cache(wb), H.make_cache(wb)
    shape = ((wb.sink_frames + 6) * wb.tokens_per_frame, wb.heads, wb.head_dim)
    q, k, v = (H.to_dev(synth.normal_bf16(shape, wb.cfg_id, 0, 9, t)) for t in "qkv")
    oa, ob = torch.empty_like(q), torch.empty_like(q)
    a.recache_prefill(0, True, 30, 6, q, k, v, oa)
    b.recache_prefill_static(0, True, 30, 6, q, k, v, ob)
    torch.cuda.synchronize()
    assert torch.equal(oa.view(torch.int16), ob.view(torch.int16))
    a.close()
    b.close()
    assert L.ll_recache_prefill_static(None, 0, 1, 3, 3, None, None, None, None, None) == B.LL_ERR_INVALID_ARG

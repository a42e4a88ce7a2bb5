"""The key set read straight out of the kernels (Sec. 3.3 "Frame Sink", "Short-window Attention").

With all queries zero every score is zero and the softmax is uniform over the key set; with V = one-hot(frame of the
token) coordinate j of the output is then (number of keys of frame j in the set) / (number of keys): 1 / |F| for the
frames of the key set F and exactly 0 for every other frame.  The expected value is a closed form, independent of
any oracle arithmetic; a key counted twice (the kblock shared by the sink and the ring is visited once per range in
the sink-relative mode), a key dropped, or a dead slot read shows up in it directly.  The oracle supplies the key
set (frames), which the host-side tests pin bit-exactly.
"""
import numpy as np
import pytest
import torch

from oracle.longlive_oracle import OracleConfig, bf16_bits_to_f64, key_frames
from paper_2509_22622_amd import binding as B
from paper_2509_22622_amd import synth

import gpu_harness as H
from test_gpu_parity import HEADS6, ODD128, ODD64

pytestmark = pytest.mark.gpu


def _one_hot_v(w, frame_ids):
    """bf16 [n*P, H, D]: row of a token of the i-th frame = unit vector e_(frame_ids[i])."""
    P = w.tokens_per_frame
    v = np.zeros((len(frame_ids) * P, w.heads, w.head_dim), np.float32)
    for i, j in enumerate(frame_ids):
        assert 0 <= j < w.head_dim
        v[i * P:(i + 1) * P, :, j] = 1.0
    return synth.f32_to_bf16_bits(v)


def _check_indicator(out, coords, what):
    """Every row of out [rows, H, D] equals 1/len(coords) on `coords` and exactly 0 elsewhere (to bf16 rounding)."""
    got = bf16_bits_to_f64(H.to_bits(out))
    want = np.zeros(got.shape[-1])
    want[list(coords)] = 1.0 / len(coords)
    off = np.ones(got.shape[-1], bool)
    off[list(coords)] = False
    assert (got[..., off] == 0.0).all(), f"{what}: weight on a frame outside the key set"
    err = np.abs(got[..., ~off] - want[~off]).max()
    assert err <= want.max() * 2.0 ** -8 * 1.01, f"{what}: {err:.3e} off 1/{len(coords)}"


def _stream_probe(w, n_chunks, sink_relative):
    cfg = OracleConfig(w.layers, w.heads, w.head_dim, w.grid_h, w.grid_w, w.chunk_frames, w.sink_frames, w.window_frames)
    cache = H.make_cache(w)
    if sink_relative:
        cache.set_sink_relative(True)
    C = w.chunk_frames
    existing = set()
    for i in range(n_chunks):
        f0 = i * C
        assert f0 + C <= w.head_dim
        shape = (w.chunk_tokens, w.heads, w.head_dim)
        q = torch.zeros(shape, dtype=torch.bfloat16, device="cuda")
        k = H.to_dev(synth.normal_bf16(shape, w.cfg_id, 0, i, "k"))
        v = H.to_dev(_one_hot_v(w, list(range(f0, f0 + C))))
        qr, out = torch.empty_like(q), torch.empty_like(q)
        cache.chunk_append(0, f0, C, q, k, v, qr)
        cache.sink_window_attn(0, qr, out)
        torch.cuda.synchronize()
        existing |= set(range(f0, f0 + C))
        F = key_frames(cfg, f0, C, existing)
        assert cache.live_frames(0) == F
        _check_indicator(out, F, f"{w.name} chunk {i} sink_relative={sink_relative}")
    cache.close()


@pytest.mark.parametrize("sink_relative", [False, True])
def test_wan_layer_streaming_reads_the_key_set(sink_relative):
    """Config 2's shape, 8 chunks: warm-up (3, 6, 9, 12 frames), steady state (15 frames) and two ring wraps; in the
    sink-relative mode the sink is a key range of its own from chunk 5 on."""
    _stream_probe(synth.WAN_LAYER, 8, sink_relative)


@pytest.mark.parametrize("w", [synth.TINY, ODD128, ODD64, HEADS6], ids=lambda w: w.name)
@pytest.mark.parametrize("sink_relative", [False, True])
def test_small_shapes_read_the_key_set(w, sink_relative):
    _stream_probe(w, min(w.n_chunks + 2, w.head_dim // w.chunk_frames), sink_relative)


@pytest.mark.parametrize("sink_relative", [False, True])
def test_recache_prefill_reads_the_chunk_causal_key_sets(sink_relative):
    """Config 5 (one layer): sink 3 + 12 window frames at a late position; chunk i of the five sees the frames of
    chunks 0 .. i and nothing else."""
    w = synth.RECACHE
    P, C, S = w.tokens_per_frame, w.chunk_frames, w.sink_frames
    ws, n_win = 165, 12
    cache = H.make_cache(w)
    if sink_relative:
        cache.set_sink_relative(True)
    n_frames = S + n_win
    shape = (n_frames * P, w.heads, w.head_dim)
    q = torch.zeros(shape, dtype=torch.bfloat16, device="cuda")
    k = H.to_dev(synth.normal_bf16(shape, w.cfg_id, 3, 7, "k"))
    v = H.to_dev(_one_hot_v(w, list(range(n_frames))))          # coordinate = position in the list of retained frames
    out = torch.empty_like(q)
    cache.recache_prefill(3, True, ws, n_win, q, k, v, out)
    torch.cuda.synchronize()
    assert cache.live_frames(3) == [0, 1, 2] + list(range(ws, ws + n_win))
    for i in range(n_frames // C):
        _check_indicator(out[i * C * P:(i + 1) * C * P], range(0, (i + 1) * C), f"cfg5 chunk {i}")
    cache.close()


def test_prefill_with_kept_sink_and_short_chunks_reads_the_key_sets():
    """include_sink = 0 after a streamed history, window not a multiple of the chunk, sink shorter than a chunk."""
    w = ODD128                                              # S 2, W 5, C 3, P 63
    P, C, S, Wn = w.tokens_per_frame, w.chunk_frames, w.sink_frames, w.window_frames
    cache = H.make_cache(w)
    shape = (w.chunk_tokens, w.heads, w.head_dim)
    for i in range(4):                                      # history: frames 0 .. 11, the sink marked 100, 101
        ids = [100 + f if f < S else 90 for f in range(i * C, (i + 1) * C)]
        cache.chunk_append(0, i * C, C, torch.zeros(shape, dtype=torch.bfloat16, device="cuda"),
                           H.to_dev(synth.normal_bf16(shape, w.cfg_id, 0, i, "k")), H.to_dev(_one_hot_v(w, ids)),
                           torch.empty(shape, dtype=torch.bfloat16, device="cuda"))
    ws, n_win = 40, 7                                       # chunks [40, 43), [43, 46), [46, 47)
    pshape = (n_win * P, w.heads, w.head_dim)
    q = torch.zeros(pshape, dtype=torch.bfloat16, device="cuda")
    out = torch.empty_like(q)
    cache.recache_prefill(0, False, ws, n_win, q, H.to_dev(synth.normal_bf16(pshape, w.cfg_id, 0, 9, "k")),
                          H.to_dev(_one_hot_v(w, list(range(n_win)))), out)
    torch.cuda.synchronize()
    row = 0
    for (a, n) in ((0, 3), (3, 3), (6, 1)):                 # window-relative frame spans of the three chunks
        lo = max(0, a - Wn)
        _check_indicator(out[row:row + n * P], [100, 101] + list(range(lo, a + n)), f"kept sink, chunk at +{a}")
        row += n * P
    cache.close()

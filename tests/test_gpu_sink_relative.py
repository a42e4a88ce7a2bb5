"""GPU parity of the variant with the sink at a fixed rotary distance (ll_cache_set_sink_relative) against
oracle/sink_relative.py, at the tolerances of the plain path (the sink's scores carry one more bf16 rounding of the
queries, which the margins of those tolerances absorb)."""
import numpy as np
import pytest
import torch

from oracle.longlive_oracle import Oracle
from oracle.sink_relative import SinkRelativeOracle
from paper_2509_22622_amd import binding as B
from paper_2509_22622_amd import synth

import gpu_harness as H
from test_gpu_parity import HEADS6, MID128, ODD128, ODD64, WIDE

pytestmark = pytest.mark.gpu


def _stream(w, n_chunks, short_last=False):
    cache, oracle, plain = H.make_cache(w), SinkRelativeOracle(H.oracle_cfg(w)), Oracle(H.oracle_cfg(w))
    cache.set_sink_relative(True)
    ref_cache = H.make_cache(w)                                        # the same stream under the plain rule
    f0, saw_shift = 0, False
    for i in range(n_chunks):
        n = 1 if (short_last and i == n_chunks - 1) else w.chunk_frames
        q, k, v = synth.chunk_qkv(w, 0, i, n)
        qd, kd, vd = H.to_dev(q), H.to_dev(k), H.to_dev(v)
        qr, out, out_plain = torch.empty_like(qd), torch.empty_like(qd), torch.empty_like(qd)
        cache.chunk_append(0, f0, n, qd, kd, vd, qr)
        cache.sink_window_attn(0, qr, out)
        ref_cache.chunk_append(0, f0, n, qd, kd, vd, qr)
        ref_cache.sink_window_attn(0, qr, out_plain)
        torch.cuda.synchronize()
        oracle.append(0, f0, q, k, v)
        plain.append(0, f0, q, k, v)
        assert cache.live_frames(0) == oracle.live_frames(0)
        H.assert_parity(H.to_bits(out), oracle.attn(0), f"{w.name} sink-relative chunk {i}")
        if oracle.delta(f0) == 0 or w.sink_frames == 0:
            assert torch.equal(out.view(torch.int16), out_plain.view(torch.int16))   # nothing differs yet
        else:
            saw_shift = True
            assert not torch.equal(out.view(torch.int16), out_plain.view(torch.int16))
            # and the difference is the variant's, not noise: the plain oracle is far from this output
            d = np.abs(H.bf16_bits_to_f64(H.to_bits(out)) - plain.attn(0)).max()
            assert d > 5 * np.abs(H.bf16_bits_to_f64(H.to_bits(out)) - oracle.attn(0)).max()
        for f in oracle.live_frames(0)[:2]:
            H.check_frame(cache, oracle, w, 0, f)                    # the cache does not depend on the setting
        f0 += n
    assert saw_shift or w.sink_frames == 0
    cache.close()
    ref_cache.close()


@pytest.mark.parametrize("w", [MID128, ODD128, ODD64, WIDE, synth.TINY], ids=lambda w: w.name)
def test_streaming_every_element(w):
    _stream(w, w.n_chunks, short_last=(w.name == "odd128"))


def _prefill(w, ws, n_win, pre_chunks=3):
    P = w.tokens_per_frame
    cache, oracle = H.make_cache(w), SinkRelativeOracle(H.oracle_cfg(w))
    cache.set_sink_relative(True)
    for i in range(pre_chunks):
        q, k, v = synth.chunk_qkv(w, 0, i)
        qd, kd, vd = H.to_dev(q), H.to_dev(k), H.to_dev(v)
        cache.chunk_append(0, i * w.chunk_frames, w.chunk_frames, qd, kd, vd, torch.empty_like(qd))
        oracle.append(0, i * w.chunk_frames, q, k, v)
    nf = w.sink_frames + n_win
    shape = (nf * P, w.heads, w.head_dim)
    q, k, v = (synth.normal_bf16(shape, w.cfg_id, 0, 500, t) for t in "qkv")
    qd, kd, vd = H.to_dev(q), H.to_dev(k), H.to_dev(v)
    out = torch.empty_like(qd)
    cache.recache_prefill(0, True, ws, n_win, qd, kd, vd, out)
    torch.cuda.synchronize()
    want = oracle.recache_prefill(0, True, ws, n_win, q, k, v)
    H.assert_parity(H.to_bits(out), want, f"{w.name} sink-relative prefill at {ws}")
    assert cache.live_frames(0) == oracle.live_frames(0)
    return H.bf16_bits_to_f64(H.to_bits(out))


def test_recache_prefill_and_invariance_under_window_position():
    """Every chunk of a re-prefill has its own shift; the same frames prefilled at another place in the video give
    the same outputs up to the rounding of the turned queries (under the plain rule they differ by far more)."""
    for w in (MID128, ODD64, HEADS6):
        n_win = w.window_frames + w.chunk_frames
        far = w.window_frames + w.sink_frames
        a = _prefill(w, far + 2, n_win)
        b = _prefill(w, far + 177, n_win)
        first = w.sink_frames * w.tokens_per_frame
        assert np.abs(a - b)[first:].max() < 6e-3                   # two bf16-rounded turnings of the same queries
        assert np.abs(a - b)[:first].max() == 0.0                   # the sink chunk itself has no shift


def test_mode_switch_and_unsupported():
    w = MID128
    cache = H.make_cache(w)
    cache.set_sink_relative(True)
    cache.set_sink_relative(False)
    c8 = B.Cache(w.layers, w.heads, w.head_dim, w.grid_h, w.grid_w, w.chunk_frames, w.sink_frames, w.window_frames,
                 kv_format="fp8_e4m3")
    with pytest.raises(B.LongLiveError) as e:
        c8.set_sink_relative(True)
    assert e.value.status == B.LL_ERR_UNSUPPORTED
    # a kernel variant without the mode: refused when a shift is due, accepted before
    cache.set_sink_relative(True)
    B.set_attn_variant(4)
    try:
        f0 = 0
        for i in range(6):
            q, k, v = synth.chunk_qkv(w, 0, i)
            qd, kd, vd = H.to_dev(q), H.to_dev(k), H.to_dev(v)
            qr, out = torch.empty_like(qd), torch.empty_like(qd)
            cache.chunk_append(0, f0, w.chunk_frames, qd, kd, vd, qr)
            if f0 <= w.window_frames + w.sink_frames:
                cache.sink_window_attn(0, qr, out)
            else:
                with pytest.raises(B.LongLiveError) as e:
                    cache.sink_window_attn(0, qr, out)
                assert e.value.status == B.LL_ERR_UNSUPPORTED
            f0 += w.chunk_frames
        torch.cuda.synchronize()
    finally:
        B.set_attn_variant(0)
    cache.close()
    c8.close()

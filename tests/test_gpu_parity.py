"""GPU parity: the HIP library through its C-ABI against the fp64 oracle, element by element."""
import numpy as np
import pytest
import torch

from oracle.longlive_oracle import Oracle, bf16_bits_to_f64
from paper_2509_22622_amd import binding as B
from paper_2509_22622_amd import synth

import gpu_harness as H

pytestmark = pytest.mark.gpu


def _stream_and_check(w, n_chunks, variant=0, q_scale=1.0, passes=1, check_cache=True, layer=0, short_last=False):
    B.set_attn_variant(variant)
    cache, oracle = H.make_cache(w), Oracle(H.oracle_cfg(w))
    worst = (0.0, 0.0)
    f0 = 0
    for i in range(n_chunks):
        n = w.chunk_frames
        if short_last and i == n_chunks - 1:
            n = 1
        for rep in range(passes):
            # all passes but the last are "noisy" versions of the chunk (Alg. 2)
            q, k, v = synth.chunk_qkv(w, layer, i + 1000 * (passes - 1 - rep), n, q_scale=q_scale)
            qd, kd, vd = H.to_dev(q), H.to_dev(k), H.to_dev(v)
            qr, out = torch.empty_like(qd), torch.empty_like(qd)
            cache.chunk_append(layer, f0, n, qd, kd, vd, qr)
            cache.sink_window_attn(layer, qr, out)
            torch.cuda.synchronize()
            q_want = oracle.append(layer, f0, q, k, v)
        assert cache.live_frames(layer) == oracle.live_frames(layer)
        H.assert_rounded(H.to_bits(qr), q_want * H.q_prescale(w), f"q' chunk {i}")
        m = H.assert_parity(H.to_bits(out), oracle.attn(layer), f"{w.name} chunk {i}", logit_scale=q_scale)
        worst = (max(worst[0], m[0]), max(worst[1], m[1]))
        if check_cache:
            for f in oracle.live_frames(layer):
                H.check_frame(cache, oracle, w, layer, f)
        f0 += n
    B.set_attn_variant(0)
    cache.close()
    return worst


def test_tiny_config_every_element():
    """Config 1: 1 layer, 4 heads x 64, 6x10 grid, chunk 3, sink 3, window 6, 8 chunks."""
    worst = _stream_and_check(synth.TINY, synth.TINY.n_chunks)
    print("tiny worst (max_abs, rel_l2):", worst)


MID128 = synth.Workload("mid128", 101, 1, 3, 128, 5, 8, 3, 3, 6, 8)       # P = 40: 8-aligned frames
ODD128 = synth.Workload("odd128", 102, 1, 2, 128, 7, 9, 3, 2, 5, 8)       # P = 63: nothing aligned, S % C != 0
NOSINK = synth.Workload("nosink", 103, 1, 2, 128, 6, 11, 2, 0, 7, 9)      # no sink, W % C != 0
ODD64 = synth.Workload("odd64", 104, 1, 3, 64, 5, 7, 3, 3, 4, 7)
WIDE = synth.Workload("wide", 105, 1, 2, 128, 16, 20, 3, 3, 3, 5)         # P = 320: several query tiles
HEADS6 = synth.Workload("heads6", 106, 1, 6, 64, 9, 15, 2, 2, 6, 8)       # P = 135: ragged tiles, many (head, chunk) groups


@pytest.mark.parametrize("w", [MID128, ODD128, NOSINK, ODD64, WIDE], ids=lambda w: w.name)
def test_small_shapes_every_element(w):
    _stream_and_check(w, w.n_chunks)


def _random_workload(rng, idx):
    """A random small geometry: nothing aligned on purpose (P from 17 to 130, any S, W, C, short last chunks)."""
    D = int(rng.choice([64, 128]))
    gh, gw = int(rng.integers(3, 11)), int(rng.integers(5, 14))
    C = int(rng.integers(1, 5))
    S = int(rng.integers(0, 6))
    Wn = int(rng.integers(0, 9))
    return synth.Workload(f"rand{idx}", 300 + idx, 1, int(rng.integers(1, 4)), D, gh, gw, C, S, Wn, int(rng.integers(4, 10)))


@pytest.mark.parametrize("idx", range(12))
def test_random_geometries_every_element(idx):
    """Seeded random (grid, chunk, sink, window, heads, head_dim): streaming with a short last chunk, every output
    element and every cached frame against the oracle, then a re-prefill of what the ring holds and two more chunks."""
    rng = np.random.default_rng(4200 + idx)
    w = _random_workload(rng, idx)
    _stream_and_check(w, w.n_chunks, short_last=bool(idx % 2))
    if w.window_frames + w.chunk_frames >= 2:
        n_win = int(rng.integers(1, w.window_frames + w.chunk_frames + 1))
        ws = w.sink_frames + int(rng.integers(0, 40))
        pre = (w.sink_frames + w.chunk_frames - 1) // w.chunk_frames + 1
        _prefill_case(w, bool(idx % 3), ws, n_win, pre_chunks=pre)


def _bf16_variants(prefix):
    """Names of the library's bf16-cache kernel variants for one head_dim (the library loads without a GPU)."""
    return [n for n in B.attn_variant_names().values()
            if n.startswith(prefix) and "fp8" not in n and "qrope" not in n]     # qrope: its own calls, tested below


def _variant_id(name):
    return {n: v for v, n in B.attn_variant_names().items()}[name]


@pytest.mark.parametrize("name", _bf16_variants("d128_"))
def test_every_d128_variant(name):
    _stream_and_check(WIDE, 5, variant=_variant_id(name), check_cache=False)
    _stream_and_check(ODD128, 6, variant=_variant_id(name), check_cache=False)


@pytest.mark.parametrize("name", _bf16_variants("d64_"))
def test_every_d64_variant(name):
    _stream_and_check(ODD64, 6, variant=_variant_id(name), check_cache=False)
    _stream_and_check(synth.TINY, 5, variant=_variant_id(name), check_cache=False)


@pytest.mark.parametrize("w", [synth.TINY, MID128, ODD128, NOSINK, ODD64, WIDE, HEADS6], ids=lambda w: w.name)
def test_unrotated_queries_bit_for_bit(w):
    """ll_chunk_append(keys and values only) + ll_sink_window_attn_unrotated against ll_chunk_append(q, q_out) +
    ll_sink_window_attn: the attention kernel turns the queries with the cache write's arithmetic, so the outputs
    agree bit for bit, and both agree with the oracle.  Several denoising passes per chunk, a short last chunk."""
    two_calls, fused, oracle = H.make_cache(w), H.make_cache(w), Oracle(H.oracle_cfg(w))
    f0, n_chunks = 0, min(w.n_chunks, 6)
    for i in range(n_chunks):
        n = 1 if i == n_chunks - 1 else w.chunk_frames
        for rep in range(2):
            q, k, v = synth.chunk_qkv(w, 0, i + 1000 * (1 - rep), n)
            qd, kd, vd = H.to_dev(q), H.to_dev(k), H.to_dev(v)
            qr, out_a, out_b = torch.empty_like(qd), torch.empty_like(qd), torch.full_like(qd, 7.0)
            two_calls.chunk_append(0, f0, n, qd, kd, vd, qr)
            two_calls.sink_window_attn(0, qr, out_a)
            fused.chunk_append(0, f0, n, None, kd, vd, None)
            fused.sink_window_attn_unrotated(0, qd, out_b)
            torch.cuda.synchronize()
            assert torch.equal(out_a.view(torch.int16), out_b.view(torch.int16)), f"{w.name} chunk {i} pass {rep}"
            oracle.append(0, f0, q, k, v)
        assert fused.live_frames(0) == oracle.live_frames(0)
        H.assert_parity(H.to_bits(out_b), oracle.attn(0), f"{w.name} chunk {i} (unrotated queries)")
        for f in oracle.live_frames(0):
            H.check_frame(fused, oracle, w, 0, f)
        f0 += n
    two_calls.close()
    fused.close()


def test_unrotated_queries_after_a_prefill_and_errors():
    """The staged chunk after ll_recache_prefill is its last chunk: ll_sink_window_attn_unrotated finds that chunk's
    frames in the middle of the table the prefill's cache write left.  Then the cases the call refuses."""
    w = ODD128
    cache = H.make_cache(w)
    P, S, C = w.tokens_per_frame, w.sink_frames, w.chunk_frames
    n_win = 5
    shape = ((S + n_win) * P, w.heads, w.head_dim)
    q, k, v = (synth.normal_bf16(shape, w.cfg_id, 0, 77, t) for t in ("q", "k", "v"))
    qd, out = H.to_dev(q), torch.empty(shape, dtype=torch.bfloat16, device="cuda")
    cache.recache_prefill(0, True, S, n_win, qd, H.to_dev(k), H.to_dev(v), out)
    # the prefill's last chunk: frames [S + n_win - last, S + n_win), rows at the tail of q
    last = n_win % C or C
    rows = slice((S + n_win - last) * P, (S + n_win) * P)
    again = torch.empty((last * P, w.heads, w.head_dim), dtype=torch.bfloat16, device="cuda")
    cache.sink_window_attn_unrotated(0, qd[rows].contiguous(), again)
    torch.cuda.synchronize()
    assert torch.equal(again.view(torch.int16), out[rows].view(torch.int16))
    # refused: a forced diagnostic variant, a re-indexed sink, an 8-bit cache, no staged chunk
    B.set_attn_variant(_variant_id("d128_stream16_tracked"))
    with pytest.raises(B.LongLiveError) as e:
        cache.sink_window_attn_unrotated(0, qd[rows].contiguous(), again)
    assert e.value.status == B.LL_ERR_UNSUPPORTED
    B.set_attn_variant(0)
    cache.reset(0)
    with pytest.raises(B.LongLiveError) as e:
        cache.sink_window_attn_unrotated(0, qd[rows].contiguous(), again)
    assert e.value.status == B.LL_ERR_STATE
    cache.close()
    c8 = B.Cache(1, w.heads, w.head_dim, w.grid_h, w.grid_w, C, S, w.window_frames, kv_format="fp8_e4m3")
    kd = H.to_dev(synth.normal_bf16((C * P, w.heads, w.head_dim), w.cfg_id, 0, 78, "k"))
    with pytest.raises(B.LongLiveError) as e:
        c8.chunk_append(0, 0, C, None, kd, kd, None)
    assert e.value.status == B.LL_ERR_UNSUPPORTED
    c8.close()


def test_peaky_softmax():
    """q scaled by 4: logits of std 4, the running reference maximum moves often."""
    _stream_and_check(MID128, 6, q_scale=4.0, check_cache=False)
    _stream_and_check(ODD64, 6, q_scale=6.0, check_cache=False)


@pytest.mark.parametrize("jump", [30.0, 200.0, 3000.0])
def test_a_late_key_far_above_the_first_kblocks_scores(jump):
    """The default kernel keeps the first kblock's maximum as its reference and only looks at the row sums at the end
    of a tile; a score far above that reference must send the tile through the pass that follows the maximum.  Keys:
    N(0,1) everywhere but one key in the fourth kblock of the second chunk that is `jump` times the query of row 5,
    normalised: that row's logit for it exceeds every other by about jump * |q| / sqrt(D) (2^200 and more as a
    weight), the other rows see it as one more random key."""
    w = MID128
    cache, oracle, marked = H.make_cache(w), Oracle(H.oracle_cfg(w)), Oracle(H.oracle_cfg(w))
    tok, v_absmax = 100, 0.0
    for i in range(3):
        q, k, v = synth.chunk_qkv(w, 0, i)
        v_marked = v
        if i == 1:
            # un-rotated key = a multiple of the un-rotated query at the same token position: the rotary step keeps them aligned
            qf = synth.bf16_bits_to_f32(q[tok, :, :])
            k[tok, :, :] = synth.f32_to_bf16_bits(qf * np.float32(jump / 8.0))
            v_marked = v.copy()
            v_marked[tok, :, :] = synth.f32_to_bf16_bits(synth.bf16_bits_to_f32(v[tok]) + np.float32(1000.0))
        qd, kd, vd = H.to_dev(q), H.to_dev(k), H.to_dev(v)
        qr, out = torch.empty_like(qd), torch.empty_like(qd)
        cache.chunk_append(0, 3 * i, 3, qd, kd, vd, qr)
        cache.sink_window_attn(0, qr, out)
        torch.cuda.synchronize()
        oracle.append(0, 3 * i, q, k, v)
        marked.append(0, 3 * i, q, k, v_marked)
        want = oracle.attn(0)
        got = bf16_bits_to_f64(H.to_bits(out))
        assert np.isfinite(got).all()
        if i == 1:
            # row `tok` of chunk 1 puts (nearly) all its weight on its own key: the output is that key's value row
            vrow = bf16_bits_to_f64(v[tok])
            if jump >= 200:
                assert np.abs(want[tok] - vrow).max() < 1e-6
                assert np.abs(got[tok] - vrow).max() <= 2.0 ** -8 * np.abs(vrow).max()
        # (row, head) pairs that give the large key no weight (the oracle's output does not move when that key's value
        # row does) are ordinary rows and must meet the graded tolerances; the others depend on a logit whose bf16
        # storage error alone exceeds them
        calm = np.abs(marked.attn(0) - want).max(axis=2) < 1e-4          # weight below 1e-7
        if i == 0:
            assert calm.all()
        if jump >= 200:
            assert calm.sum() > calm.size // 8
        if calm.any():
            H.assert_parity(H.to_bits(out)[calm], want[calm], f"late dominant key x{jump}, chunk {i}")
        # and every output, calm or not, is a convex combination of value rows
        v_absmax = max(v_absmax, np.abs(bf16_bits_to_f64(v)).max())
        assert np.abs(got).max() <= v_absmax * (1 + 2.0 ** -7)
    cache.close()


@pytest.mark.parametrize("q_scale", [16.0, 64.0, 256.0])
def test_extreme_logits_stay_finite_and_convex(q_scale):
    """Logits of std 16 to 256 (softmax close to one-hot, the reference maximum jumps by far more than the slack in
    almost every kblock).  bf16 storage of q' and k' moves such logits by more than 1, so element-wise parity is not
    defined; what holds at any scale: outputs are finite, every output lies in the convex hull of the V rows of the
    key set (per head and feature), and rows with a dominant key reproduce that key's V."""
    w = WIDE
    cache, oracle = H.make_cache(w), Oracle(H.oracle_cfg(w))
    for i in range(4):
        q, k, v = synth.chunk_qkv(w, 0, i, q_scale=q_scale)
        qd, kd, vd = H.to_dev(q), H.to_dev(k), H.to_dev(v)
        qr, out = torch.empty_like(qd), torch.empty_like(qd)
        cache.chunk_append(0, 3 * i, 3, qd, kd, vd, qr)
        cache.sink_window_attn(0, qr, out)
        torch.cuda.synchronize()
        oracle.append(0, 3 * i, q, k, v)
        got = bf16_bits_to_f64(H.to_bits(out))
        assert np.isfinite(got).all(), f"chunk {i}"
        vals = np.concatenate([oracle.frame_kv(0, f)[1] for f in oracle.live_frames(0)])      # [keys, H, D]
        lo, hi = vals.min(axis=0), vals.max(axis=0)
        tol = 2.0 ** -7 * np.maximum(np.abs(lo), np.abs(hi))                                   # output rounding
        assert (got >= lo - tol).all() and (got <= hi + tol).all(), f"chunk {i}: output outside the hull of V"
        want = oracle.attn(0)
        # rows whose softmax is decided (the oracle's largest weight dominates) must agree closely
        err = np.abs(got - want).max(axis=-1)
        agree = (err < 0.05).mean()
        assert agree > 0.5, f"chunk {i}: only {agree:.2f} of the (row, head) outputs near the oracle"
    cache.close()


def test_only_the_last_pass_stays():
    """Alg. 2: several passes of a chunk at the same start frame, the last one is what later chunks see."""
    _stream_and_check(MID128, 6, passes=3)


def test_dead_slots_may_hold_nan():
    """A frame that left the key set but still sits in a ring slot must have no influence, even as NaN."""
    w = ODD128
    cache, oracle = H.make_cache(w), Oracle(H.oracle_cfg(w))
    f0 = 0
    n_chunks = 7
    for i in range(n_chunks):
        n = 1 if i == n_chunks - 1 else w.chunk_frames                 # a short chunk leaves dead frames behind
        q, k, v = synth.chunk_qkv(w, 0, i, n)
        if i == 3:                                                      # poison this chunk's K and V
            k = np.full_like(k, 0x7FC0)
            v = np.full_like(v, 0x7FC0)
        qd, kd, vd = H.to_dev(q), H.to_dev(k), H.to_dev(v)
        qr, out = torch.empty_like(qd), torch.empty_like(qd)
        cache.chunk_append(0, f0, n, qd, kd, vd, qr)
        cache.sink_window_attn(0, qr, out)
        torch.cuda.synchronize()
        oracle.append(0, f0, q, k, v)
        live = oracle.live_frames(0)
        assert cache.live_frames(0) == live
        poisoned_live = any(9 <= f < 12 for f in live)
        if not poisoned_live:
            H.assert_parity(H.to_bits(out), oracle.attn(0), f"chunk {i}")
        f0 += n
    # the last chunk was short: frames of the poisoned chunk are dead but not yet overwritten
    assert not any(9 <= f < 12 for f in live)
    assert cache.slot_of_frame(0, 11) not in [cache.slot_of_frame(0, f) for f in live]
    cache.close()


def _prefill_case(w, include_sink, ws, n_win, pre_chunks, follow=2, variant=0):
    B.set_attn_variant(variant)
    P = w.tokens_per_frame
    cache, oracle = H.make_cache(w), Oracle(H.oracle_cfg(w))
    for i in range(pre_chunks):                                         # some history first
        q, k, v = synth.chunk_qkv(w, 0, i)
        qd, kd, vd = H.to_dev(q), H.to_dev(k), H.to_dev(v)
        cache.chunk_append(0, i * w.chunk_frames, w.chunk_frames, qd, kd, vd, torch.empty_like(qd))
        oracle.append(0, i * w.chunk_frames, q, k, v)
    nf = (w.sink_frames if include_sink else 0) + n_win
    shape = (nf * P, w.heads, w.head_dim)
    q, k, v = (synth.normal_bf16(shape, w.cfg_id, 0, 500, t) for t in "qkv")
    qd, kd, vd = H.to_dev(q), H.to_dev(k), H.to_dev(v)
    out = torch.empty_like(qd)
    cache.recache_prefill(0, include_sink, ws, n_win, qd, kd, vd, out)
    torch.cuda.synchronize()
    want = oracle.recache_prefill(0, include_sink, ws, n_win, q, k, v)
    H.assert_parity(H.to_bits(out), want, f"{w.name} prefill")
    assert cache.live_frames(0) == oracle.live_frames(0)
    for f in oracle.live_frames(0):
        H.check_frame(cache, oracle, w, 0, f)
    f0 = ws + n_win
    for i in range(follow):                                             # streaming goes on from the rebuilt cache
        q, k, v = synth.chunk_qkv(w, 0, 600 + i)
        qd, kd, vd = H.to_dev(q), H.to_dev(k), H.to_dev(v)
        qr, out = torch.empty_like(qd), torch.empty_like(qd)
        cache.chunk_append(0, f0, w.chunk_frames, qd, kd, vd, qr)
        cache.sink_window_attn(0, qr, out)
        torch.cuda.synchronize()
        oracle.append(0, f0, q, k, v)
        assert cache.live_frames(0) == oracle.live_frames(0)
        H.assert_parity(H.to_bits(out), oracle.attn(0), f"{w.name} after prefill {i}")
        f0 += w.chunk_frames
    B.set_attn_variant(0)
    cache.close()


def test_recache_prefill_small():
    _prefill_case(MID128, True, 3, 9, pre_chunks=4)                     # window right after the sink
    _prefill_case(MID128, True, 177, 9, pre_chunks=60)                  # late window, ring wrapped many times
    _prefill_case(MID128, False, 15, 9, pre_chunks=8)                   # sink kept as it is
    _prefill_case(ODD128, True, 8, 7, pre_chunks=5)                     # S % C != 0, short last chunk
    _prefill_case(ODD64, True, 12, 6, pre_chunks=6)
    _prefill_case(NOSINK, True, 10, 9, pre_chunks=10)                   # no sink at all
    _prefill_case(HEADS6, True, 20, 8, pre_chunks=4)                    # 6 heads x 5 chunks: groups placed XCD by XCD
    _prefill_case(HEADS6, False, 31, 7, pre_chunks=6)


def test_prefill_equals_streaming_on_the_gpu():
    """Same q,k,v streamed chunk by chunk or prefilled at once: same outputs, same cache bits."""
    w = MID128
    P, nf = w.tokens_per_frame, 12
    shape = (nf * P, w.heads, w.head_dim)
    q, k, v = (synth.normal_bf16(shape, w.cfg_id, 0, 700, t) for t in "qkv")
    qd, kd, vd = H.to_dev(q), H.to_dev(k), H.to_dev(v)
    a, b = H.make_cache(w), H.make_cache(w)
    outs = []
    for f0 in range(0, nf, 3):
        sl = slice(f0 * P, (f0 + 3) * P)
        qr, o = torch.empty_like(qd[sl]), torch.empty_like(qd[sl])
        a.chunk_append(0, f0, 3, qd[sl], kd[sl], vd[sl], qr)
        a.sink_window_attn(0, qr, o)
        outs.append(o)
    ob = torch.empty_like(qd)
    b.recache_prefill(0, True, 3, 9, qd, kd, vd, ob)
    torch.cuda.synchronize()
    assert torch.equal(torch.cat(outs).view(torch.int16), ob.view(torch.int16))
    assert a.live_frames(0) == b.live_frames(0) and a.live_ranges(0) == b.live_ranges(0)
    for f in a.live_frames(0):
        ka, va, kb, vb = (torch.empty((P, w.heads, w.head_dim), dtype=torch.bfloat16, device="cuda") for _ in range(4))
        a.read_frame(0, f, ka, va)
        b.read_frame(0, f, kb, vb)
        torch.cuda.synchronize()
        assert torch.equal(ka.view(torch.int16), kb.view(torch.int16)) and torch.equal(va.view(torch.int16), vb.view(torch.int16))
    a.close()
    b.close()


def test_deterministic_and_in_place():
    """Two runs give identical bits; q_out may alias q and out may alias q_roped."""
    w = WIDE
    q, k, v = synth.chunk_qkv(w, 0, 0)
    res = []
    for rep in range(2):
        cache = H.make_cache(w)
        qd, kd, vd = H.to_dev(q), H.to_dev(k), H.to_dev(v)
        if rep == 0:
            qr, out = torch.empty_like(qd), torch.empty_like(qd)
            cache.chunk_append(0, 0, 3, qd, kd, vd, qr)
            cache.sink_window_attn(0, qr, out)
        else:
            cache.chunk_append(0, 0, 3, qd, kd, vd, qd)
            cache.sink_window_attn(0, qd, qd)
            out = qd
        torch.cuda.synchronize()
        res.append(H.to_bits(out))
        cache.close()
    assert np.array_equal(res[0], res[1])


def test_device_argument_errors():
    """Errors that need a device handle: null and misaligned tensors, attention without a staged chunk, aliasing in
    the prefill.  Nothing is enqueued by a failing call; the handle stays usable."""
    w = MID128
    cache = H.make_cache(w)
    n = w.chunk_tokens * w.heads * w.head_dim
    shape = (w.chunk_tokens, w.heads, w.head_dim)
    base = torch.zeros(n + 8, dtype=torch.bfloat16, device="cuda")
    good, odd = base[:n].view(shape), base[1:n + 1].view(shape)        # odd starts 2 bytes into the allocation
    assert odd.data_ptr() % 16 == 2
    out = torch.empty_like(good)
    with pytest.raises(B.LongLiveError) as e:
        cache.sink_window_attn(0, good, out)                            # nothing staged yet
    assert e.value.status == B.LL_ERR_STATE
    with pytest.raises(B.LongLiveError) as e:
        cache.chunk_append(0, 0, w.chunk_frames, odd, good, good, out)
    assert e.value.status == B.LL_ERR_INVALID_ARG and "aligned" in str(e.value)
    assert cache.live_frames(0) == []                                   # the failed append changed nothing
    with pytest.raises(B.LongLiveError) as e:
        cache.chunk_append(0, 0, w.chunk_frames, good, good, None, out)
    assert e.value.status == B.LL_ERR_INVALID_ARG
    cache.chunk_append(0, 0, w.chunk_frames, good, good, good, out)
    with pytest.raises(B.LongLiveError) as e:
        cache.sink_window_attn(0, out, odd)
    assert e.value.status == B.LL_ERR_INVALID_ARG
    nf = w.sink_frames + 3
    big = torch.zeros((nf * w.tokens_per_frame, w.heads, w.head_dim), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(B.LongLiveError) as e:
        cache.recache_prefill(0, True, w.sink_frames, 3, big, big, big, big)     # out aliases the inputs
    assert e.value.status == B.LL_ERR_INVALID_ARG
    cache.sink_window_attn(0, out, torch.empty_like(out))               # still usable
    torch.cuda.synchronize()
    cache.close()


MANY = synth.Workload("many-chunks", 107, 1, 2, 64, 3, 5, 1, 2, 40, 6)     # chunk = 1 frame, ring of 41 frames


def test_prefill_beyond_one_launch():
    """A re-prefill of 43 frames in chunks of one frame: more frames than one append launch takes (32) and more
    chunks than one attention launch takes (16), so the library cuts both; streaming goes on afterwards."""
    _prefill_case(MANY, True, 50, 41, pre_chunks=4, follow=3)
    _prefill_case(MANY, False, 7, 20, pre_chunks=3, follow=2)           # 20 chunks: two attention launches


def test_read_frame_one_tensor_at_a_time():
    """ll_cache_read_frame with only k_out or only v_out (either may be NULL) returns the same bits as with both."""
    w = ODD128
    cache = H.make_cache(w)
    q, k, v = synth.chunk_qkv(w, 0, 0)
    qd = H.to_dev(q)
    cache.chunk_append(0, 0, w.chunk_frames, qd, H.to_dev(k), H.to_dev(v), torch.empty_like(qd))
    shape = (w.tokens_per_frame, w.heads, w.head_dim)
    both_k, both_v, only_k, only_v = (torch.zeros(shape, dtype=torch.bfloat16, device="cuda") for _ in range(4))
    for frame in range(w.chunk_frames):
        cache.read_frame(0, frame, both_k, both_v)
        cache.read_frame(0, frame, only_k, None)
        cache.read_frame(0, frame, None, only_v)
        torch.cuda.synchronize()
        assert torch.equal(both_k.view(torch.int16), only_k.view(torch.int16)), frame
        assert torch.equal(both_v.view(torch.int16), only_v.view(torch.int16)), frame
        P = w.tokens_per_frame
        assert np.array_equal(H.to_bits(only_v), v[frame * P:(frame + 1) * P])      # V is stored bit-exact
    cache.close()


@pytest.mark.parametrize("ws", [60000, 2 ** 31 + 77])
def test_prefill_and_streaming_at_very_late_frames(ws):
    """Frame indices are 64-bit and absolute: the rotary angles of the frame axis are taken in fp64 on the device, so a
    window hours into a video (or past 2^31 frames) is as exact as one at the start."""
    _prefill_case(ODD64, True, ws, ODD64.window_frames + ODD64.chunk_frames, pre_chunks=3)

"""The prompt side of KV-recache on the GPU (ll_prompt_recache, ll_cross_attn) against the fp64 oracle.

Tolerances: relative L2 as for the self-attention path (5e-3).  The outputs are convex combinations of a few value
rows and as large as the values themselves, so the absolute bound of the benchmark definition (1e-2, made for outputs
of size 0.01 to 0.1) is scaled by max(1, max|v|): rounding an output near 4 to bf16 alone moves it by up to 2^-7.
"""
import numpy as np
import pytest
import torch

from oracle.longlive_oracle import bf16_bits_to_f64, error_metrics
from oracle.prompt_cross_attention import PromptOracle, cross_attention
from paper_2509_22622_amd import binding as B
from paper_2509_22622_amd import synth

import gpu_harness as H

pytestmark = pytest.mark.gpu

CFG = 31        # stream id of these inputs in the seeded generator


def bits(shape, stream, tensor, scale=1.0):
    return synth.normal_bf16(shape, CFG, 0, stream, tensor, scale=scale)


def assert_parity_prompt(out_bits, want, v_bits, what):
    got = bf16_bits_to_f64(out_bits)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    max_abs, rel = error_metrics(got, want)
    bound = H.MAX_ABS_TOL * max(1.0, float(np.abs(bf16_bits_to_f64(v_bits)).max()))
    assert max_abs <= bound and rel <= H.REL_L2_TOL, f"{what}: max_abs {max_abs:.3e} (bound {bound:.3e}) rel_l2 {rel:.3e}"
    return max_abs, rel


@pytest.mark.parametrize("heads,head_dim,n_q,n_t", [
    (4, 64, 300, 1), (4, 64, 300, 31), (4, 64, 300, 32), (4, 64, 300, 33), (4, 64, 1, 77), (4, 64, 257, 77),
    (3, 128, 1000, 512), (2, 128, 513, 100), (12, 128, 700, 226),
])
def test_cross_attn_parity(heads, head_dim, n_q, n_t):
    p = B.Prompt(2, heads, head_dim, 512)
    oracle = PromptOracle(2, heads, head_dim)
    for layer, stream in ((1, 3), (0, 4)):                 # two layers with different prompts
        k, v = bits((n_t, heads, head_dim), stream, "k"), bits((n_t, heads, head_dim), stream, "v")
        p.recache(layer, H.to_dev(k), H.to_dev(v))
        oracle.recache(layer, bf16_bits_to_f64(k), bf16_bits_to_f64(v))
    assert p.tokens(0) == n_t and p.tokens(1) == n_t
    for layer in (0, 1):
        q = bits((n_q, heads, head_dim), 5 + layer, "q")
        out = torch.empty((n_q, heads, head_dim), dtype=torch.bfloat16, device="cuda")
        p.cross_attn(layer, H.to_dev(q), out)
        torch.cuda.synchronize()
        want = oracle.cross_attn(layer, bf16_bits_to_f64(q))
        assert_parity_prompt(H.to_bits(out), want, bits((n_t, heads, head_dim), 3 if layer == 1 else 4, "v"),
                             f"layer {layer} H{heads} D{head_dim} n_q {n_q} n_t {n_t}")
    p.close()


def _scaling_variants(head_dim):
    """Kernel variants that apply the factor log2(e)/sqrt(D) themselves: the ones ll_cross_attn accepts."""
    return [n for n in B.attn_variant_names().values()
            if n.startswith(f"d{head_dim}_") and "fp8" not in n and (n.endswith("_qscale") or "_q" in n)]


@pytest.mark.parametrize("name", _scaling_variants(128) + _scaling_variants(64))
def test_every_kernel_variant_the_call_accepts(name):
    """ll_cross_attn picks a kernel by the launch's size; here each candidate is forced in turn (and a variant that
    expects pre-scaled queries, if selected, is ignored rather than used)."""
    heads, head_dim, n_q, n_t = 3, int(name[1:name.index("_")]), 700, 226
    ids = {n: v for v, n in B.attn_variant_names().items()}
    q, k, v = bits((n_q, heads, head_dim), 30, "q"), bits((n_t, heads, head_dim), 30, "k"), bits((n_t, heads, head_dim), 30, "v")
    p = B.Prompt(1, heads, head_dim, 256)
    p.recache(0, H.to_dev(k), H.to_dev(v))
    want = cross_attention(bf16_bits_to_f64(q), bf16_bits_to_f64(k), bf16_bits_to_f64(v))
    try:
        for forced in (name, f"d{head_dim}_stream"):
            B.set_attn_variant(ids[forced])
            out = torch.empty((n_q, heads, head_dim), dtype=torch.bfloat16, device="cuda")
            p.cross_attn(0, H.to_dev(q), out)
            torch.cuda.synchronize()
            assert_parity_prompt(H.to_bits(out), want, v, f"variant {forced}")
    finally:
        B.set_attn_variant(0)
    p.close()


@pytest.mark.parametrize("head_dim", [64, 128])
def test_values_and_keys_stay_paired_bit_exact(head_dim):
    """Keys 40 e_j and queries 40 e_i: query i puts all its weight on token i (the others get 2^-288, zero in
    fp32), so the output must be token i's value row bit for bit: the keys went into the cache unchanged, each next
    to its own value, across several 32-token blocks."""
    heads, n_t = 2, head_dim
    k = np.zeros((n_t, heads, head_dim), dtype=np.float32)
    for j in range(n_t):
        k[j, :, (j * 7) % head_dim] = 40.0                  # 7 is coprime to D: a permutation of the axes
    kb = synth.f32_to_bf16_bits(k)
    vb = bits((n_t, heads, head_dim), 8, "v")
    q = np.zeros((3 * n_t, heads, head_dim), dtype=np.float32)
    for i in range(3 * n_t):
        q[i, :, ((i % n_t) * 7) % head_dim] = 40.0
    p = B.Prompt(1, heads, head_dim, n_t)
    p.recache(0, H.to_dev(kb), H.to_dev(vb))
    out = torch.empty(q.shape, dtype=torch.bfloat16, device="cuda")
    p.cross_attn(0, H.to_dev(synth.f32_to_bf16_bits(q)), out)
    torch.cuda.synchronize()
    got = H.to_bits(out)
    for i in range(3 * n_t):
        assert np.array_equal(got[i], vb[i % n_t]), f"query {i}"
    p.close()


def test_one_token_prompt_returns_its_value_bit_exact():
    heads, head_dim, n_q = 3, 128, 290
    kb, vb = bits((1, heads, head_dim), 9, "k", 5.0), bits((1, heads, head_dim), 9, "v")
    p = B.Prompt(1, heads, head_dim, 16)
    p.recache(0, H.to_dev(kb), H.to_dev(vb))
    out = torch.empty((n_q, heads, head_dim), dtype=torch.bfloat16, device="cuda")
    p.cross_attn(0, H.to_dev(bits((n_q, heads, head_dim), 10, "q", 3.0)), out)
    torch.cuda.synchronize()
    assert np.array_equal(H.to_bits(out), np.broadcast_to(vb, (n_q, heads, head_dim)))
    p.close()


def test_switch_to_a_shorter_prompt_leaves_no_trace():
    """Sec. 3.1: after the switch the state belongs to the new prompt alone.  The former prompt is longer and its
    keys are large (they would take all the weight if any of them were still read)."""
    heads, head_dim, n_q = 4, 64, 400
    q = bits((n_q, heads, head_dim), 11, "q")
    k_old, v_old = bits((77, heads, head_dim), 12, "k", 30.0), bits((77, heads, head_dim), 12, "v", 8.0)
    k_new, v_new = bits((40, heads, head_dim), 13, "k"), bits((40, heads, head_dim), 13, "v")
    used, fresh = B.Prompt(1, heads, head_dim, 128), B.Prompt(1, heads, head_dim, 128)
    out_old, out_used, out_fresh = (torch.empty((n_q, heads, head_dim), dtype=torch.bfloat16, device="cuda") for _ in range(3))
    used.recache(0, H.to_dev(k_old), H.to_dev(v_old))
    used.cross_attn(0, H.to_dev(q), out_old)
    used.recache(0, H.to_dev(k_new), H.to_dev(v_new))
    used.cross_attn(0, H.to_dev(q), out_used)
    fresh.recache(0, H.to_dev(k_new), H.to_dev(v_new))
    fresh.cross_attn(0, H.to_dev(q), out_fresh)
    torch.cuda.synchronize()
    assert used.tokens(0) == 40
    assert torch.equal(out_used.view(torch.int16), out_fresh.view(torch.int16))
    assert not torch.equal(out_used.view(torch.int16), out_old.view(torch.int16))
    want = cross_attention(bf16_bits_to_f64(q), bf16_bits_to_f64(k_new), bf16_bits_to_f64(v_new))
    assert_parity_prompt(H.to_bits(out_used), want, v_new, "after the switch")
    used.close()
    fresh.close()


@pytest.mark.parametrize("forced", [None, "d128_q1x4_k1_occ3"])
def test_output_over_the_queries(forced):
    heads, head_dim, n_q, n_t = 4, 128, 600, 90
    q, k, v = bits((n_q, heads, head_dim), 14, "q"), bits((n_t, heads, head_dim), 14, "k"), bits((n_t, heads, head_dim), 14, "v")
    p = B.Prompt(1, heads, head_dim, 128)
    p.recache(0, H.to_dev(k), H.to_dev(v))
    qd = H.to_dev(q)
    out = torch.empty_like(qd)
    try:
        if forced:
            B.set_attn_variant({n: i for i, n in B.attn_variant_names().items()}[forced])
        p.cross_attn(0, qd, out)
        p.cross_attn(0, qd, qd)                             # in place
        torch.cuda.synchronize()
    finally:
        B.set_attn_variant(0)
    assert torch.equal(qd.view(torch.int16), out.view(torch.int16))
    p.close()


def test_peaky_scores():
    """Queries four times larger: logits of standard deviation 4, a few tokens carry the weight."""
    heads, head_dim, n_q, n_t = 4, 128, 520, 512
    q, k, v = bits((n_q, heads, head_dim), 15, "q", 4.0), bits((n_t, heads, head_dim), 15, "k"), bits((n_t, heads, head_dim), 15, "v")
    p = B.Prompt(1, heads, head_dim, 512)
    p.recache(0, H.to_dev(k), H.to_dev(v))
    out = torch.empty((n_q, heads, head_dim), dtype=torch.bfloat16, device="cuda")
    p.cross_attn(0, H.to_dev(q), out)
    torch.cuda.synchronize()
    want = cross_attention(bf16_bits_to_f64(q), bf16_bits_to_f64(k), bf16_bits_to_f64(v))
    got = bf16_bits_to_f64(H.to_bits(out))
    max_abs, rel = error_metrics(got, want)
    # logits four times larger: the rounding of q' and k to bf16 moves them four times further (the same allowance
    # as the self-attention path's stress input)
    assert rel <= 4 * H.REL_L2_TOL and max_abs <= 4 * H.MAX_ABS_TOL * 4.5, f"max_abs {max_abs:.3e} rel_l2 {rel:.3e}"
    p.close()


@pytest.mark.parametrize("n_q", [4680, 23400])
def test_wan_shape_full_size(n_q):
    """The benchmark model's shape: 12 heads of 128, 512 prompt tokens; the queries of one chunk (4680) and of one
    re-prefill (23400).  Every output element is compared."""
    heads, head_dim, n_t, layers = 12, 128, 512, 2
    p = B.Prompt(layers, heads, head_dim, n_t)
    k, v = bits((n_t, heads, head_dim), 16, "k"), bits((n_t, heads, head_dim), 16, "v")
    q = bits((n_q, heads, head_dim), 17, "q")
    p.recache(1, H.to_dev(k), H.to_dev(v))
    out = torch.empty((n_q, heads, head_dim), dtype=torch.bfloat16, device="cuda")
    p.cross_attn(1, H.to_dev(q), out)
    torch.cuda.synchronize()
    want = cross_attention(bf16_bits_to_f64(q), bf16_bits_to_f64(k), bf16_bits_to_f64(v))
    assert_parity_prompt(H.to_bits(out), want, v, f"wan shape n_q {n_q}")
    p.close()


@pytest.mark.parametrize("heads,head_dim,n_q,n_t", [
    (12, 128, 11000, 256), (12, 64, 12345, 512), (5, 128, 40000, 768), (12, 128, 11000, 250), (12, 128, 11000, 200),
])
def test_many_query_tiles(heads, head_dim, n_q, n_t):
    """Launches of more than two rounds of query tiles (the small-workgroup kernel): 8, 16, 24 kblocks of keys, a
    partly dead last kblock, ragged last query tiles, both head sizes.  Every output element against the oracle."""
    p = B.Prompt(1, heads, head_dim, 1024)
    k, v = bits((n_t, heads, head_dim), 41, "k"), bits((n_t, heads, head_dim), 41, "v")
    q = bits((n_q, heads, head_dim), 42, "q")
    p.recache(0, H.to_dev(k), H.to_dev(v))
    out = torch.full((n_q, heads, head_dim), 3.0, dtype=torch.bfloat16, device="cuda")
    p.cross_attn(0, H.to_dev(q), out)
    torch.cuda.synchronize()
    want = cross_attention(bf16_bits_to_f64(q), bf16_bits_to_f64(k), bf16_bits_to_f64(v))
    assert_parity_prompt(H.to_bits(out), want, v, f"H{heads} D{head_dim} n_q {n_q} n_t {n_t}")
    p.close()


def test_graph_replay_of_a_prompt_switch():
    """Both calls enqueue kernels only: captured in a graph, a replay re-runs the switch and the cross-attention on
    what the captured tensors hold now."""
    heads, head_dim, n_q, n_t = 4, 64, 300, 77
    eager, graphed = B.Prompt(1, heads, head_dim, 128), B.Prompt(1, heads, head_dim, 128)
    sk, sv = (torch.zeros((n_t, heads, head_dim), dtype=torch.bfloat16, device="cuda") for _ in range(2))
    sq = torch.zeros((n_q, heads, head_dim), dtype=torch.bfloat16, device="cuda")
    sout = torch.empty_like(sq)

    def one(p, q, k, v, out):
        p.recache(0, k, v)
        p.cross_attn(0, q, out)

    one(graphed, sq, sk, sv, sout)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        one(graphed, sq, sk, sv, sout)
    for rep in range(3):
        q, k, v = bits(sq.shape, 20 + rep, "q"), bits(sk.shape, 20 + rep, "k"), bits(sk.shape, 20 + rep, "v")
        out = torch.empty_like(sq)
        one(eager, H.to_dev(q), H.to_dev(k), H.to_dev(v), out)
        torch.cuda.synchronize()
        sq.copy_(H.to_dev(q)), sk.copy_(H.to_dev(k)), sv.copy_(H.to_dev(v))
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(sout.view(torch.int16), out.view(torch.int16)), f"replay {rep}"
        want = cross_attention(bf16_bits_to_f64(q), bf16_bits_to_f64(k), bf16_bits_to_f64(v))
        assert_parity_prompt(H.to_bits(sout), want, v, f"replay {rep}")
    eager.close()
    graphed.close()


# ---- the block's output path: attention over the prompt, then the layer's output projection (ll_cross_attn_out)

def _weight(heads, head_dim, stream):
    """bf16 weight [H*D, H*D], N(0, 1 / (H*D)): the projection keeps the size of its input."""
    n = heads * head_dim
    return synth.normal_bf16((n, n), CFG, 0, stream, "k", scale=1.0 / np.sqrt(n))


def assert_parity_projection(y_bits, want, v_bits, what):
    """Relative L2 as everywhere (5e-3): y inherits the attention output's error (its bf16 rounding included: the
    projection reads the rounded tensor, the oracle the exact one), adds fp32 summation noise and one more bf16
    rounding (2^-9 relative, about 1.1e-3 in relative L2).  Absolute bound scaled like the attention output's."""
    got = bf16_bits_to_f64(y_bits)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    max_abs, rel = error_metrics(got, want)
    bound = H.MAX_ABS_TOL * max(1.0, float(np.abs(bf16_bits_to_f64(v_bits)).max()))
    assert max_abs <= bound and rel <= H.REL_L2_TOL, f"{what}: max_abs {max_abs:.3e} (bound {bound:.3e}) rel_l2 {rel:.3e}"


def _project(p, q_dev, w_dev, y=None):
    """ll_cross_attn_out with a freshly packed weight and a workspace of exactly the size the library asks for."""
    n_q, n = q_dev.shape[0], p.heads * p.head_dim
    w_packed = torch.empty_like(w_dev)
    p.pack_out_weight(w_dev, w_packed)
    nbytes = p.cross_attn_out_workspace_bytes(n_q)
    assert nbytes == (n_q + 15) // 16 * 16 * n * 2
    work = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    if y is None:
        y = torch.full((n_q, n), 9.0, dtype=torch.bfloat16, device="cuda")
    p.cross_attn_out(0, q_dev, w_packed, work, y)
    return y


@pytest.mark.parametrize("heads,head_dim,n_q,n_t", [
    (4, 64, 300, 33), (3, 64, 1, 5), (3, 64, 129, 77),          # N = 256, 192 (one and a half weight blocks), ragged rows
    (3, 128, 1000, 512), (2, 128, 513, 100), (12, 128, 700, 226), (5, 128, 257, 40),
])
def test_cross_attn_out_parity(heads, head_dim, n_q, n_t):
    from oracle.prompt_cross_attention import cross_attention_out
    p = B.Prompt(1, heads, head_dim, 512)
    k, v = bits((n_t, heads, head_dim), 11, "k"), bits((n_t, heads, head_dim), 11, "v")
    q = bits((n_q, heads, head_dim), 12, "q")
    w = _weight(heads, head_dim, 13)
    p.recache(0, H.to_dev(k), H.to_dev(v))
    y = _project(p, H.to_dev(q), H.to_dev(w))
    torch.cuda.synchronize()
    want = cross_attention_out(bf16_bits_to_f64(q), bf16_bits_to_f64(k), bf16_bits_to_f64(v), bf16_bits_to_f64(w))
    assert_parity_projection(H.to_bits(y), want, v, f"H{heads} D{head_dim} n_q {n_q} n_t {n_t}")
    p.close()


@pytest.mark.parametrize("heads,head_dim,n_q,n_t", [(3, 128, 300, 50), (5, 64, 77, 50),
                                                    (12, 128, 11000, 50), (12, 64, 11000, 50),    # many query tiles: the small-workgroup kernel
                                                    (12, 128, 11000, 256), (12, 64, 11000, 256)])
def test_out_projection_exact_cases(heads, head_dim, n_q, n_t):
    """Weights the projection must pass through bit for bit: the identity returns the attention output itself (what
    ll_cross_attn writes: so the hand-over between the two kernels loses and moves nothing), a permutation moves its
    features."""
    n = heads * head_dim
    p = B.Prompt(1, heads, head_dim, 256)
    k, v, q = bits((n_t, heads, head_dim), 21, "k"), bits((n_t, heads, head_dim), 21, "v"), bits((n_q, heads, head_dim), 22, "q")
    p.recache(0, H.to_dev(k), H.to_dev(v))
    qd = H.to_dev(q)
    attn = torch.empty((n_q, heads, head_dim), dtype=torch.bfloat16, device="cuda")
    p.cross_attn(0, qd, attn)
    eye = torch.eye(n, dtype=torch.bfloat16, device="cuda")
    y = _project(p, qd, eye)
    torch.cuda.synchronize()
    assert torch.equal(y.view(torch.int16), attn.reshape(n_q, n).view(torch.int16))
    perm = torch.from_numpy(np.random.default_rng(5).permutation(n)).cuda()
    pw = torch.zeros((n, n), dtype=torch.bfloat16, device="cuda")
    pw[torch.arange(n, device="cuda"), perm] = 1.0                      # y[:, j] = x[:, perm[j]]
    y = _project(p, qd, pw)
    torch.cuda.synchronize()
    assert torch.equal(y.view(torch.int16), attn.reshape(n_q, n)[:, perm].contiguous().view(torch.int16))
    p.close()


def test_cross_attn_out_refuses_overlapping_tensors():
    heads, head_dim, n_q = 2, 64, 40
    n = heads * head_dim
    p = B.Prompt(1, heads, head_dim, 64)
    kv = H.to_dev(bits((9, heads, head_dim), 21, "k"))
    p.recache(0, kv, kv)
    qd = H.to_dev(bits((n_q, heads, head_dim), 22, "q"))
    w = torch.eye(n, dtype=torch.bfloat16, device="cuda")
    wp = torch.empty_like(w)
    p.pack_out_weight(w, wp)
    work = torch.empty(p.cross_attn_out_workspace_bytes(n_q), dtype=torch.uint8, device="cuda")
    y = torch.empty((n_q, n), dtype=torch.bfloat16, device="cuda")
    for args in ((qd, wp, y, y), (qd, wp, qd, y), (qd, wp, work, qd), (qd, wp, wp, y)):
        with pytest.raises(B.LongLiveError) as e:
            p.cross_attn_out(0, *args)
        assert e.value.status == B.LL_ERR_INVALID_ARG
    with pytest.raises(B.LongLiveError) as e:
        p.pack_out_weight(w, w)
    assert e.value.status == B.LL_ERR_INVALID_ARG
    p.close()


def test_cross_attn_out_benchmark_shape():
    """12 heads x 128, 512 prompt tokens, a chunk's 4680 queries: every element of the projected output."""
    from oracle.prompt_cross_attention import cross_attention_out
    heads, head_dim, n_q, n_t = 12, 128, 4680, 512
    p = B.Prompt(1, heads, head_dim, 512)
    k, v = bits((n_t, heads, head_dim), 31, "k"), bits((n_t, heads, head_dim), 31, "v")
    q, w = bits((n_q, heads, head_dim), 32, "q"), _weight(heads, head_dim, 33)
    p.recache(0, H.to_dev(k), H.to_dev(v))
    y = _project(p, H.to_dev(q), H.to_dev(w))
    torch.cuda.synchronize()
    want = cross_attention_out(bf16_bits_to_f64(q), bf16_bits_to_f64(k), bf16_bits_to_f64(v), bf16_bits_to_f64(w))
    assert_parity_projection(H.to_bits(y), want, v, "benchmark shape")
    p.close()

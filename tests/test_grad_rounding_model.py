"""Where the gradient tolerances of tests/test_gpu_clip.py come from: a rounding model of the backward path on the CPU.

The model is the oracle's backward (oracle/clip_backward.py: same formulas, fp64) with a rounding to bf16 at each place
where the GPU path rounds, and nowhere else:
    q'   the rotated, pre-scaled queries as the cache-write kernel stores them      (enters the logits)
    K'   the rotated keys as stored                                                 (enters the logits and the dQ product)
    Pf   the forward's weights before its second product                            (enters delta through the output)
    P    the weights rebuilt in the backward, operand of the dV product
    dZ   = P (dP - delta), operand of the dQ and dK products
    out  the final rounding of dq, dk, dv
Everything else (fp32 accumulation, exp2, the fp32 copy of the forward's output that delta is taken from) is exact
here; those errors are 2^-24-sized.  One rounding of unit roundoff u = 2^-8 (bf16 keeps 8 significant bits) is uniform
within +-u/2 of a value's binade, i.e. at most rho = u / sqrt(3) = 2.26e-3 in relative L2 (measured below: 1.66e-3 for
normal data, whose significands are spread over the binade).  A gradient tensor sees n_r such roundings on its way
    dq: q' and K' in the logits, dZ, K' as the product's operand, the result      n_r = 5
    dk: q' and K' in the logits, dZ, q' as the product's operand, the result      n_r = 5
    dv: q' and K' in the logits, P, the result                                    n_r = 4
and, their errors being independent and every sum running over many terms, they add in quadrature:
    relative L2 <= sqrt(n_r) * rho = 5.0e-3 (dq, dk), 4.5e-3 (dv).
(The roundings inside the logits count a little less than one each: the softmax removes their weighted mean.)  Where
nothing averages (a handful of keys, one of them holding the weight) a rounding can sit at its maximum u instead of
its root mean square: sqrt(n_r) * u = 8.7e-3 and 7.8e-3; and no single element can be off by more than n_r * u = 2 %
of the tensor's largest magnitude.  This file checks on the CPU that the model behaves as this arithmetic says; the
GPU tests then hold the kernels to the same bounds.
"""
import math

import numpy as np
import pytest

from oracle.clip_backward import ClipOracle, _unrotate_grad
from oracle.longlive_oracle import OracleConfig, bf16_bits_to_f64, error_metrics, key_frames, rope_rotate
from paper_2509_22622_amd import synth

U_BF16 = 2.0 ** -8
RHO = U_BF16 / math.sqrt(3.0)
N_ROUNDINGS = {"dq": 5, "dk": 5, "dv": 4}
PLACES = ("q", "k", "pf", "p", "dz", "out")


def round_bf16(x):
    """Round to nearest even at 8 significant bits, through fp32 (every value here is far inside fp32's range)."""
    bits = np.asarray(x, dtype=np.float32).view(np.uint32)
    bits = (bits + np.uint32(0x7FFF) + ((bits >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return bits.view(np.float32).astype(np.float64)


def rounded_backward(cfg, ctx_start, n_ctx, n_clip, q, k, v, dout, places=PLACES):
    """The oracle's forward and backward with bf16 roundings at `places` (module docstring)."""
    P, D = cfg.tokens_per_frame, cfg.head_dim
    oracle = ClipOracle(cfg)
    frames = oracle.frames(ctx_start, n_ctx, n_clip)
    pos = {f: i for i, f in enumerate(frames)}
    clip_start = ctx_start + n_ctx
    r = lambda place, x: round_bf16(x) if place in places else x
    c = math.log2(math.e) / math.sqrt(D)                      # the stored queries carry this factor; scores are log2
    k_rot = r("k", np.concatenate([rope_rotate(cfg, k[pos[f] * P:(pos[f] + 1) * P], f) for f in frames]))
    q_rot = r("q", rope_rotate(cfg, q, clip_start) * c)
    dq_rot, dk_rot, dv_all = np.zeros_like(q_rot), np.zeros_like(k_rot), np.zeros_like(v)
    for f0, n in oracle.clip_chunks(clip_start, n_clip):
        keys = key_frames(cfg, f0, n, [f for f in frames if f < f0 + n])
        kidx = np.concatenate([np.arange(pos[f] * P, (pos[f] + 1) * P) for f in keys])
        rows = slice((f0 - clip_start) * P, (f0 - clip_start + n) * P)
        for h in range(cfg.heads):
            s2 = q_rot[rows, h] @ k_rot[kidx, h].T
            m = s2.max(axis=1, keepdims=True)
            w = np.exp2(s2 - m)
            l = w.sum(axis=1, keepdims=True)
            out = (r("pf", w) @ v[kidx, h]) / l               # the forward's output, kept unrounded for delta
            p = np.exp2(s2 - (m + np.log2(l)))
            do = dout[rows, h]
            dz = p * (do @ v[kidx, h].T - (do * out).sum(axis=1, keepdims=True))
            dv_all[kidx, h] += r("p", p).T @ do
            dq_rot[rows, h] = (r("dz", dz) @ k_rot[kidx, h]) / math.sqrt(D)
            dk_rot[kidx, h] += (r("dz", dz).T @ q_rot[rows, h]) * math.log(2.0)
    first = pos[clip_start] * P
    return {"dq": r("out", _unrotate_grad(cfg, dq_rot, clip_start)),
            "dk": r("out", _unrotate_grad(cfg, dk_rot[first:], clip_start)),
            "dv": r("out", dv_all[first:])}


def _inputs(cfg, ctx_start, n_ctx, n_clip, seed):
    P, H, D = cfg.tokens_per_frame, cfg.heads, cfg.head_dim
    nf = len(ClipOracle(cfg).frames(ctx_start, n_ctx, n_clip))
    f = lambda shape, stream, tensor: bf16_bits_to_f64(synth.normal_bf16(shape, 41, 0, stream, tensor))
    return (f((n_clip * P, H, D), 4 * seed, "q"), f((nf * P, H, D), 4 * seed, "k"), f((nf * P, H, D), 4 * seed, "v"),
            f((n_clip * P, H, D), 4 * seed + 1, "q"))


def _errors(cfg, ctx_start, n_ctx, n_clip, seed, places):
    q, k, v, dout = _inputs(cfg, ctx_start, n_ctx, n_clip, seed)
    oracle = ClipOracle(cfg)
    oracle.forward(ctx_start, n_ctx, n_clip, q, k, v)
    want = dict(zip(("dq", "dk", "dv"), oracle.backward(dout)))
    got = rounded_backward(cfg, ctx_start, n_ctx, n_clip, q, k, v, dout, places)
    return {name: error_metrics(got[name], want[name])[1] for name in want}


CASES = [(OracleConfig(1, 2, 64, 4, 5, 3, 3, 9), 12, 9, 6), (OracleConfig(1, 2, 128, 4, 5, 3, 3, 9), 12, 9, 6)]


def test_without_roundings_the_model_is_the_oracle():
    cfg, ctx_start, n_ctx, n_clip = CASES[0]
    err = _errors(cfg, ctx_start, n_ctx, n_clip, 0, places=())
    assert max(err.values()) < 1e-12, err


@pytest.mark.parametrize("case", range(len(CASES)))
def test_one_rounding_is_at_most_rho(case):
    """Each place alone: no more than rho per use, and the final rounding (one use, nothing in front of it) shows the
    root mean square of a single rounding."""
    cfg, ctx_start, n_ctx, n_clip = CASES[case]
    uses = {"q": {"dq": 1, "dk": 2, "dv": 1}, "k": {"dq": 2, "dk": 1, "dv": 1}, "pf": {"dq": 1, "dk": 1, "dv": 0},
            "p": {"dq": 0, "dk": 0, "dv": 1}, "dz": {"dq": 1, "dk": 1, "dv": 0}, "out": {"dq": 1, "dk": 1, "dv": 1}}
    for place in PLACES:
        err = _errors(cfg, ctx_start, n_ctx, n_clip, 0, places=(place,))
        for name, e in err.items():
            assert e <= math.sqrt(uses[place][name]) * RHO + 1e-12, f"{place} -> {name}: {e:.3e}"
        if place == "out":
            assert all(0.6 * RHO <= e <= RHO for e in err.values()), err
        if place == "pf":                                     # the forward's rounded weights reach delta only
            assert max(err.values()) < 0.2 * RHO, err


@pytest.mark.parametrize("case", range(len(CASES)))
def test_all_roundings_add_in_quadrature_below_the_gate(case):
    cfg, ctx_start, n_ctx, n_clip = CASES[case]
    alone = {place: _errors(cfg, ctx_start, n_ctx, n_clip, 0, places=(place,)) for place in PLACES}
    full = _errors(cfg, ctx_start, n_ctx, n_clip, 0, places=PLACES)
    for name, e in full.items():
        quad = math.sqrt(sum(alone[place][name] ** 2 for place in PLACES))
        assert abs(e - quad) <= 0.05 * quad, f"{name}: {e:.3e} against {quad:.3e} in quadrature"
        gate = math.sqrt(N_ROUNDINGS[name]) * RHO
        assert 0.5 * gate <= e <= gate, f"{name}: {e:.3e} outside [{0.5 * gate:.3e}, {gate:.3e}]"

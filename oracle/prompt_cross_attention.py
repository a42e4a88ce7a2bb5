"""CPU oracle for the prompt side of KV-recache: cross-attention of video tokens over the active prompt's keys.

TEST INFRASTRUCTURE ONLY.  Plain fp64 numpy; only tests, the smoke check and the bench's ``cpu_baseline`` leg may
import it.  It shares no code with the HIP path and imports nothing from the product package.

What it follows: Sec. 3.1 "KV Recache" and Fig. 2 (right).  In the DiT the self-attention layers alternate with
cross-attention layers through which the prompt enters; at a prompt switch the cached state is rebuilt from the
frames generated so far *paired with the new prompt*.  On the self-attention side that is the chunk-causal re-prefill
(``longlive_oracle.Oracle.recache_prefill``); on the cross-attention side the per-layer keys and values projected from
the prompt's embeddings are replaced by those of the new prompt, and every later cross-attention (the re-prefill's
own and all following chunks') reads the new ones only.  The attention itself is the textbook definition: no mask,
no positional embedding on either side, every query sees every prompt token.

Readings (the paper gives no formulas for this layer): scale 1/sqrt(D); the prompt's length may differ from one
prompt to the next and tokens of an earlier, longer prompt must leave no trace; the projections that produce q, k and
v belong to the model and are inputs here.

The layer's output path (Fig. 2, right: the cross-attention block's result goes back into the video tokens' stream)
is the plain output projection of a multi-head attention: the heads' outputs of a token are concatenated and
multiplied by the layer's output weight, y = concat_heads(o) W^T with W [H*D, H*D] stored as a linear layer stores it
([output feature][input feature]).  No bias here (a bias is an addition the caller can make); the weight belongs to
the model and is an input.

Pins (tests/test_oracle_pins.py): loops on tiny inputs, a library's scaled-dot-product attention, closed forms (one
token; equal keys give the mean of the values; a dominant key), invariance under a permutation of the prompt's
tokens, and independence from the replaced prompt; for the output projection: scalar loops, a library's linear
layer, the identity weight (returns the concatenated heads), a permutation weight (moves features, bit for bit),
linearity, and a weight that reads one head only.
"""
from __future__ import annotations

import math

import numpy as np


def cross_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray) -> np.ndarray:
    """softmax(q k^T / sqrt(D)) v per head.  q [Nq, H, D]; k, v [Nt, H, D]; returns [Nq, H, D] float64."""
    q, k, v = (np.asarray(a, dtype=np.float64) for a in (q, k, v))
    nq, heads, d = q.shape
    assert k.shape == v.shape and k.shape[1:] == (heads, d) and k.shape[0] >= 1
    out = np.empty((nq, heads, d))
    for h in range(heads):
        s = (q[:, h, :] @ k[:, h, :].T) / math.sqrt(d)            # [Nq, Nt]
        s -= s.max(axis=1, keepdims=True)
        w = np.exp(s)
        w /= w.sum(axis=1, keepdims=True)
        out[:, h, :] = w @ v[:, h, :]
    return out


def out_projection(o: np.ndarray, w: np.ndarray) -> np.ndarray:
    """y[t, n] = sum over (h, d) of o[t, h, d] * w[n, h * D + d].  o [Nq, H, D]; w [H*D, H*D]; returns [Nq, H*D]."""
    o, w = np.asarray(o, dtype=np.float64), np.asarray(w, dtype=np.float64)
    nq, heads, d = o.shape
    assert w.shape == (heads * d, heads * d)
    return o.reshape(nq, heads * d) @ w.T


def cross_attention_out(q, k, v, w) -> np.ndarray:
    """The cross-attention block's output: attention over the prompt, then the output projection."""
    return out_projection(cross_attention(q, k, v), w)


class PromptOracle:
    """The prompt-side state of all layers: one (k, v) pair per layer, replaced as a whole at a prompt switch."""

    def __init__(self, layers: int, heads: int, head_dim: int):
        self.layers, self.heads, self.head_dim = layers, heads, head_dim
        self._kv = [None] * layers

    def recache(self, layer: int, k: np.ndarray, v: np.ndarray) -> None:
        k, v = np.array(k, dtype=np.float64), np.array(v, dtype=np.float64)
        assert k.shape == v.shape and k.shape[1:] == (self.heads, self.head_dim) and k.shape[0] >= 1
        self._kv[layer] = (k, v)                                   # nothing of the former prompt is kept

    def tokens(self, layer: int) -> int:
        return 0 if self._kv[layer] is None else self._kv[layer][0].shape[0]

    def cross_attn(self, layer: int, q: np.ndarray) -> np.ndarray:
        if self._kv[layer] is None:
            raise RuntimeError(f"layer {layer}: no prompt")
        return cross_attention(q, *self._kv[layer])
